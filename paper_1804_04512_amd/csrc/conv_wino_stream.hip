// Forward pass of a padded 3x3 layer with 16 channels in and 16 filters behind ReLU + 2x2 max pooling
// (Section II-A, valid convolution; Section IV-B, pooling), in the minimal-filtering form F(2x2, 3x3)
//   Y = At [ (G g Gt) .* (Bt d B) ] A   per 2x2 block of outputs and its 4x4 input patch,
// as a wavefront-private streaming kernel on fp32 MFMA (v_mfma_f32_16x16x4_f32), gfx950.
//
// Per transform point p the sums over the input channels are a matrix product,
// M_p[block][k] = sum_c V_p[block][c] U_p[c][k]: blocks on the MFMA M axis, filters on N, channels
// on K.  Lane (i16, kq) transforms the patch of block i16 of the wavefront's 16-block row segment for
// the channels kq, 4+kq, 8+kq, 12+kq (its A fragments) and ends up with all 16 point sums of the
// blocks 4kq .. 4kq+3 for filter i16, so both transforms are register-local; a 2x2 block is one
// pooling window, so bias, ReLU, maximum and position follow in registers and only the pooled row
// (16 bytes per lane) and its pooling bytes (4 per lane) are stored.  The transformed filters - 64
// values per lane - stay in registers for the whole kernel.
//
// Every wavefront works alone: its own 32-column segment, its own four-row ring of image rows in LDS
// (two new rows per block row), no workgroup barrier after the filters are in place.  Rows travel from
// memory through two register sets in turn and are requested two block rows ahead of their use,
// straight across work-item boundaries; every block row issues the same loads and stores on every
// path (out-of-range offsets where there is nothing to move), so the number of memory instructions
// issued after any given one is known at compile time and a wait leaves the later ones in flight.
#include "conv_wgrad_wino_body.h"
#include "dll_internal.h"

#include <type_traits>

namespace dllk {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;
constexpr int kRS = 36;                 // LDS row: image columns x0-1 .. x0+32 at LDS columns 0 .. 33
constexpr int kPS = 4 * kRS + 2;        // channel plane of four row slots
constexpr int kWaveFloats = 16 * kPS;   // one wavefront's ring: 16 channels
constexpr int kXR = 4;                  // 16 channels x 2 rows x 8 aligned 16-byte groups = 4 per lane
constexpr unsigned kOob = 0x80000000u;

struct WinoStreamParams {
  ConvEngineArgs a;
  int Hp, Wp;          // pooled map = blocks per column / row
  int xsegs, xgroups;  // 32-pixel column segments; groups of as many neighbouring segments as a workgroup has streams
  int rg, rgroups;     // block rows per work item, row groups per image
  int items;           // work items of a workgroup: N * rgroups * xgroups
  int G;               // workgroups
  unsigned x_bytes, y_bytes;
};

// KT: groups of 16 filters (1 or 2); a wavefront works ONE group (with two groups, two wavefronts stage
// the same rows, each into its own ring).
// CH: halves of a 32-channel source (1: 16 channels).  With CH = 2 two wavefronts work the two halves of
// the same segment and filter group; after the output transform (it is linear) the wavefront of the
// upper half hands its 16 values per lane over through LDS and the other adds them and finishes.  That
// costs one workgroup barrier per packet, so with CH = 2 all four wavefronts run the same packets in
// step: no wavefront skips an item (the launcher takes only shapes whose segments fill the streams).
// The 4 / (KT * CH) remaining wavefronts are independent streams over neighbouring segments.
template <bool IDX, int KT, int CH>
__global__ __launch_bounds__(kThreads, 2) void conv3x3_wino_stream_kernel(const WinoStreamParams p) {
  extern __shared__ float lds[];
  const ConvEngineArgs &a = p.a;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same in every lane: it lives in scalar registers
  const int i16 = lane & 15, kq = lane >> 4;
  const int gidx = blockIdx.x;
  constexpr int S = 4 / (KT * CH), kKout = 16 * KT, kCin = 16 * CH;
  const int chalf = wave % CH, ktile = (wave / CH) % KT, stream = wave / (CH * KT);
  const int c0 = 16 * chalf, k0 = 16 * ktile;
  float *xs = lds + wave * kWaveFloats;
  floatx4 *exch = reinterpret_cast<floatx4 *>(lds + 4 * kWaveFloats);   // CH = 2: [packet parity][pair][4][lane]

  // ---- transformed filters U = G g Gt, G = [1 0 0; .5 .5 .5; .5 -.5 .5; 0 0 1]: per (channel half, filter
  // group), one (channel, filter) pair per thread into LDS [point][channel][filter] (over the rings, which
  // are not in use yet); the wavefronts of that half and group then take their B fragments: channel
  // 4s+kq, filter i16, every point
  float U[4][16];
#pragma unroll
  for (int cb = 0; cb < CH * KT; ++cb) {
    const int ch = cb % CH, kt = cb / CH;
    {
      const int c = tid >> 4, k = tid & 15;
      const float *g = a.w + ((long)(16 * kt + k) * kCin + 16 * ch + c) * 9;
      float gv[9];
#pragma unroll
      for (int e = 0; e < 9; ++e) gv[e] = g[e];
      float t[4][3];
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        t[0][j] = gv[j];
        t[1][j] = 0.5f * (gv[j] + gv[3 + j] + gv[6 + j]);
        t[2][j] = 0.5f * (gv[j] - gv[3 + j] + gv[6 + j]);
        t[3][j] = gv[6 + j];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        lds[((4 * i + 0) * 16 + c) * 16 + k] = t[i][0];
        lds[((4 * i + 1) * 16 + c) * 16 + k] = 0.5f * (t[i][0] + t[i][1] + t[i][2]);
        lds[((4 * i + 2) * 16 + c) * 16 + k] = 0.5f * (t[i][0] - t[i][1] + t[i][2]);
        lds[((4 * i + 3) * 16 + c) * 16 + k] = t[i][2];
      }
    }
    __syncthreads();
    if (ch == chalf && kt == ktile) {
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int q = 0; q < 16; ++q) U[s][q] = lds[(q * 16 + 4 * s + kq) * 16 + i16];
    }
    __syncthreads();   // everybody has its fragments: the next group, or the rings, may be written
  }
  const float bias = a.bias ? a.bias[k0 + i16] : 0.0f;

  const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.src), 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, (int)p.y_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_i = __builtin_amdgcn_make_buffer_rsrc(a.out_idx, 0, IDX ? (int)(p.y_bytes >> 2) : 0, 0x00020000);

  // Staging slots of a pair of image rows.  Main slots: (channel, row of the pair, aligned 16-byte
  // group j of the segment), four per lane; halo slots: (channel, row, left or right neighbour
  // column), one per lane.  A slot's place in the tensor is fixed per work item (xv, hv: byte
  // offsets of the slot in the item's FIRST pair, or an out-of-range offset where the slot lies
  // outside the image: such loads return zero, the padding value).
  int xlo[kXR], xcol[kXR], xpl[kXR];
  bool xr1[kXR];
#pragma unroll
  for (int it = 0; it < kXR; ++it) {
    const int s = lane + 64 * it;
    const int ch = s >> 4, rr = (s >> 3) & 1, j = s & 7;
    xr1[it] = rr == 1;
    xpl[it] = (ch * a.Hin + rr) * a.Win + 4 * j;      // elements from (n, channel 0, first row of the pair, x0)
    xcol[it] = 4 * j;
    xlo[it] = ch * kPS + rr * kRS + 4 * j + 1;
  }
  const int h_ch = lane >> 2, h_rr = (lane >> 1) & 1, h_side = lane & 1;
  const int hpl = (h_ch * a.Hin + h_rr) * a.Win + (h_side ? 32 : -1);
  const int hlo = h_ch * kPS + h_rr * kRS + (h_side ? 33 : 0);

  float4 xa[kXR], xb[kXR];   // two pairs of rows on their way from memory to LDS
  float ha = 0.0f, hb = 0.0f;
  unsigned xv[kXR], hv = kOob;   // byte offsets of the lane's slots in the first pair of the item being requested

  auto item_setup = [&](int n, int x0, int by0) {
    const int base = ((n * kCin + c0) * a.Hin + (2 * by0 - 1)) * a.Win + x0;
#pragma unroll
    for (int it = 0; it < kXR; ++it) xv[it] = x0 + xcol[it] < a.Win ? 4u * (unsigned)(base + xpl[it]) : kOob;
    const int hc = x0 + (h_side ? 32 : -1);
    hv = (x0 < a.Win && (unsigned)hc < (unsigned)a.Win) ? 4u * (unsigned)(base + hpl) : kOob;
  };
  // rows 2P-1 and 2P -> registers; dP = P - by0 of the item.  The pair's distance from the item's
  // first pair is added to the lanes' offsets, not passed as the loads' scalar offset: row -1 of the
  // tensor's very first plane has a negative offset, and the range check of a buffer load looks at
  // the vector offset on its own, so a negative one made good by a scalar offset would read zero.
  auto load_pair = [&](int P, int dP, float4 (&xr)[kXR], float &xh) {
    const unsigned down = (unsigned)(8 * a.Win) * (unsigned)dP;
    const bool top = P == 0, bot = 2 * P >= a.Hin;      // the pair's first row is above / its second row below the image
#pragma unroll
    for (int it = 0; it < kXR; ++it) {
      unsigned off = xv[it] + down;                     // an out-of-range marker stays one (down < 2^24)
      if (top || bot) off = (xr1[it] ? bot : top) ? kOob : off;
      const floatx4 v = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rs_x, (int)off, 0, 0));
      xr[it] = make_float4(v[0], v[1], v[2], v[3]);
    }
    unsigned off = hv + down;
    if (top || bot) off = (h_rr ? bot : top) ? kOob : off;
    xh = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_x, (int)off, 0, 0));
  };
  // registers -> the pair's two row slots (image column x0 sits at LDS column 1)
  auto store_pair = [&](int slotpair, const float4 (&xr)[kXR], float xh) {
    float *dst = xs + slotpair * 2 * kRS;
#pragma unroll
    for (int it = 0; it < kXR; ++it) {
      float *d = dst + xlo[it];
      d[0] = xr[it].x;
      *reinterpret_cast<float2 *>(d + 1) = make_float2(xr[it].y, xr[it].z);
      d[3] = xr[it].w;
    }
    dst[hlo] = xh;
  };

  // ---- one block row of the segment: 16 blocks x 16 filters; `sp` = parity of the block row inside its
  // item = which row slots hold its upper pair of rows (the lower pair sits in the other two).
  // `yo`: element offset of the lane's four pooled outputs (filter i16, blocks 4kq .. 4kq+3), or out of range.
  const float *patch = xs + kq * kPS + 2 * i16;
  const floatx4 zero = {0.f, 0.f, 0.f, 0.f};
  // The input transform V = Bt d B is taken row-wise first: H = d B for each image row (four
  // values per row and lane), then V = Bt H down the four rows of a patch.  Patches of neighbouring
  // block rows share two rows, and the wavefront walks downwards: the H of a packet's two rows is
  // computed once, when the packet arrives (`Hn`), serves as the lower half of the block row that
  // is worked then and, kept in registers (`Hp` of the next packet), as the upper half of the next
  // one.  24 instead of 32 additions and two instead of four row reads per patch and channel quartet.
  // The two H sets swap roles from packet to packet like the two register sets of the packets.
  auto h_row = [&](const float2 &l, const float2 &h, float (&o)[4]) {
    o[0] = l.x - h.x;
    o[1] = l.y + h.x;
    o[2] = h.x - l.y;
    o[3] = l.y - h.y;
  };
  // a packet that brings the first pair of rows of an item: only its H is taken
  auto prime = [&](int slot, float (&Hn)[4][2][4]) {
    const float *pnew = patch + slot * 2 * kRS;
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        const float *row = pnew + r * kRS + 4 * s * kPS;
        h_row(*reinterpret_cast<const float2 *>(row), *reinterpret_cast<const float2 *>(row + 2), Hn[s][r]);
      }
  };
  auto block_row = [&](int slot, const float (&Hp)[4][2][4], float (&Hn)[4][2][4], floatx4 (&z)[4]) {
    const float *pnew = patch + slot * 2 * kRS;   // the packet just stored: the block row's lower pair of rows
    floatx4 acc[16];
    float2 pl[2][2], ph[2][2];
    auto read_patch = [&](auto sc) {
      constexpr int s = decltype(sc)::value;
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        const float *row = pnew + r * kRS + 4 * s * kPS;
        pl[s & 1][r] = *reinterpret_cast<const float2 *>(row);
        ph[s & 1][r] = *reinterpret_cast<const float2 *>(row + 2);
      }
    };
    auto quartet = [&](auto sc) {
      constexpr int s = decltype(sc)::value;
      if constexpr (s < 3) read_patch(std::integral_constant<int, s + 1>{});
      __builtin_amdgcn_sched_barrier(0);
      h_row(pl[s & 1][0], ph[s & 1][0], Hn[s][0]);
      h_row(pl[s & 1][1], ph[s & 1][1], Hn[s][1]);
      // ---- V = Bt H, Bt = [1 0 -1 0; 0 1 1 0; 0 -1 1 0; 0 1 0 -1], rows: Hp[0], Hp[1], Hn[0], Hn[1]
      float V[16];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        V[j] = Hp[s][0][j] - Hn[s][0][j];
        V[4 + j] = Hp[s][1][j] + Hn[s][0][j];
        V[8 + j] = Hn[s][0][j] - Hp[s][1][j];
        V[12 + j] = Hp[s][1][j] - Hn[s][1][j];
      }
      // the whole transform first, then the 16 products back to back (a switch between vector and
      // matrix instructions costs about eight cycles each time)
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(V[q], U[s][q], s == 0 ? zero : acc[q], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    };
    read_patch(std::integral_constant<int, 0>{});
    quartet(std::integral_constant<int, 0>{});
    quartet(std::integral_constant<int, 1>{});
    quartet(std::integral_constant<int, 2>{});
    quartet(std::integral_constant<int, 3>{});
    // ---- output transform At M A, At = [1 1 1 0; 0 1 -1 -1]: z[v] = the 2x2 block 4kq+v (y00, y01, y10, y11)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      float sr[2][4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        sr[0][j] = acc[j][v] + acc[4 + j][v] + acc[8 + j][v];
        sr[1][j] = acc[4 + j][v] - acc[8 + j][v] - acc[12 + j][v];
      }
      z[v] = floatx4{sr[0][0] + sr[0][1] + sr[0][2], sr[0][1] - sr[0][2] - sr[0][3],
                     sr[1][0] + sr[1][1] + sr[1][2], sr[1][1] - sr[1][2] - sr[1][3]};
    }
  };
  // bias, ReLU, pooling: a block is one window; first maximum in the order (0,0), (0,1), (1,0), (1,1)
  auto finish = [&](const floatx4 (&z)[4], floatx4 &y, unsigned &ib) {
    float yv[4];
    ib = 0;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      float m = z[v][0];
      unsigned arg = 0;
      if (z[v][1] > m) { m = z[v][1]; arg = 1; }
      if (z[v][2] > m) { m = z[v][2]; arg = 2; }
      if (z[v][3] > m) { m = z[v][3]; arg = 3; }
      const float o = m + bias;
      yv[v] = o > 0.0f ? o : 0.0f;
      ib |= (arg | (yv[v] > 0.0f ? 0u : (unsigned)kIdxInactive)) << (8 * v);
    }
    y = floatx4{yv[0], yv[1], yv[2], yv[3]};
  };

  // ---- work items: (image, group of block rows, group of four neighbouring column segments), one
  // segment per wavefront, so that the wavefronts of a workgroup read neighbouring pieces of the same
  // image rows at about the same time; each wavefront walks its segment downwards.  A wavefront whose
  // segment lies beyond the row (the last group of a row that is not a multiple of four segments
  // wide) skips the item.  Packet q of an item of n block rows (q = 0 .. n) is the pair of image rows
  // 2(by0+q)-1, 2(by0+q); handling it means moving it into the ring (row slots 2(q&1), 2(q&1)+1), asking
  // for the packet after next into the register set just emptied, and (q >= 1) working block row q-1,
  // whose upper pair the packet before brought.
  auto rows_of = [&](int item, int &n_img, int &xseg, int &by0) -> int {
    const int xg = item % p.xgroups;
    const int rgrp = (item / p.xgroups) % p.rgroups;
    n_img = item / (p.xgroups * p.rgroups);
    xseg = xg * S + stream;
    by0 = rgrp * p.rg;
    // (CH = 2: never skipped, the four wavefronts stay in step; a segment beyond the row would be worked on zeros)
    return (CH == 2 || xseg < p.xsegs) ? min(by0 + p.rg, p.Hp) - by0 : 0;
  };
  // request cursor: packet (r_item, r_q) is the next to ask for; consume cursor: (c_item, c_q) the next to handle
  int r_item = gidx - p.G, r_q = 0, r_n = -1, r_by0 = 0;
  auto next_request_item = [&]() {
    int n_img = 0, xseg = 0;
    r_n = 0;
    for (r_item += p.G; r_item < p.items; r_item += p.G)
      if ((r_n = rows_of(r_item, n_img, xseg, r_by0)) > 0) break;
    r_q = 0;
    if (r_item < p.items) {
      item_setup(n_img, xseg * 32, r_by0);
    } else {                                      // nothing left: every further request reads zeros
#pragma unroll
      for (int it = 0; it < kXR; ++it) xv[it] = kOob;
      hv = kOob;
      r_by0 = 0;
    }
  };
  auto request = [&](float4 (&xr)[kXR], float &xh) {
    load_pair(r_by0 + r_q, r_q, xr, xh);
    if (++r_q > r_n) next_request_item();
  };
  int c_item = gidx - p.G, c_q = 0, c_n = -1, c_par = 0;
  unsigned c_yo = kOob;   // element offset of the lane's outputs in the item's first block row
  auto next_consume_item = [&]() {
    int n_img = 0, xseg = 0, by0 = 0;
    c_n = 0;
    for (c_item += p.G; c_item < p.items; c_item += p.G)
      if ((c_n = rows_of(c_item, n_img, xseg, by0)) > 0) break;
    c_q = 0;
    const int bx = xseg * 16 + 4 * kq;
    c_yo = (c_item < p.items && bx < p.Wp) ? (unsigned)(((n_img * kKout + k0 + i16) * p.Hp + by0) * p.Wp + bx) : kOob;
  };
  // (a packet handled after the wavefront's last item is an empty one: the loop below leaves only after
  // whole rounds of both register sets, so that no path leads from one set's packet straight to the
  // same set's next - the compiler would have to assume the loads just issued are the ones awaited)
  auto handle = [&](float4 (&xr)[kXR], float &xh, const float (&Hp)[4][2][4], float (&Hn)[4][2][4]) {
    const bool live = c_item < p.items;
    store_pair(c_q & 1, xr, xh);
    request(xr, xh);
    // the stores are issued for every packet (out of range where no block row was worked), like the loads
    floatx4 z[4] = {zero, zero, zero, zero};
    floatx4 y = zero;
    unsigned ib = 0, yo = kOob;
    const bool work = live && c_q > 0;
    if (work) block_row(c_q & 1, Hp, Hn, z);
    else prime(c_q & 1, Hn);
    if constexpr (CH == 2) {
      // the upper half's partial blocks go to the lower half's wavefront; every wavefront of the
      // workgroup passes this barrier once per packet
      floatx4 *ex = exch + ((c_par * 2 + wave / 2) * 4) * 64 + lane;
      if (chalf == 1) {
#pragma unroll
        for (int v = 0; v < 4; ++v) ex[64 * v] = z[v];
      }
      __syncthreads();
      if (chalf == 0) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const floatx4 o = ex[64 * v];
          z[v] += o;
        }
      }
      c_par ^= 1;
    }
    if (work && chalf == 0) {
      finish(z, y, ib);
      if (c_yo != kOob) yo = c_yo + (unsigned)((c_q - 1) * p.Wp);
    }
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uintx4, y), rs_y, (int)(yo == kOob ? kOob : 4u * yo), 0, 0);
    if (IDX) __builtin_amdgcn_raw_buffer_store_b32(ib, rs_i, (int)yo, 0, 0);
    if (live && ++c_q > c_n) next_consume_item();
  };

  next_request_item();
  next_consume_item();
  // the first two requests, each followed by the (empty) stores of a packet, so that the loop is entered
  // with the same sequence of memory instructions behind it as one of its own rounds leaves
  auto empty_stores = [&]() {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uintx4, zero), rs_y, (int)kOob, 0, 0);
    if (IDX) __builtin_amdgcn_raw_buffer_store_b32(0u, rs_i, (int)kOob, 0, 0);
  };
  request(xa, ha);
  empty_stores();
  request(xb, hb);
  empty_stores();
  float H0[4][2][4] = {}, H1[4][2][4] = {};
  while (c_item < p.items) {
    handle(xa, ha, H0, H1);
    handle(xb, hb, H1, H0);
  }
}

// ---- Backward-data pass of such a layer (the full convolution of Section II-A as a valid one with
// rotated, transposed filters): the source is dz = unpool(dy) with the ReLU flags of the pooling
// bytes, formed in the ring from the pooled gradient; the 2x2 output blocks are stored as they are.
//
// A packet is one POOLED row of the segment: 16 channels x (16 + 2 neighbour) gradients and pooling
// bytes; handling it writes the two dz rows of its windows into one of three slot pairs of a six-row
// ring (pooled row R of an item starting at block row by0 sits in slot pair (R - by0 + 1) mod 3).
// Block row by needs dz rows 2by-1 .. 2by+2: the lower row of pooled row by-1, both rows of pooled
// row by, the upper row of pooled row by+1; an item of n block rows therefore has n + 2 packets.
constexpr int kPSB = 6 * kRS + 2;        // channel plane of six row slots; half of it odd
constexpr int kWaveFloatsB = 16 * kPSB;

// KT: groups of 16 output channels, CH: halves of a 32-channel gradient, as in the forward kernel.
// (the body as a function of the workgroup's index `gidx` among p.G workgroups and its dynamic LDS: it
// also runs as one role of the launch it shares with the layer's filter gradient, below)
template <int KT, int CH>
__device__ __forceinline__ void stream_bwd_body(const WinoStreamParams &p, float *lds, const int gidx) {
  const ConvEngineArgs &a = p.a;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i16 = lane & 15, kq = lane >> 4;
  constexpr int S = 4 / (KT * CH), kKout = 16 * KT, kCin = 16 * CH;
  const int chalf = wave % CH, ktile = (wave / CH) % KT, stream = wave / (CH * KT);
  const int c0 = 16 * chalf, k0 = 16 * ktile;
  float *xs = lds + wave * kWaveFloatsB;
  floatx4 *exch = reinterpret_cast<floatx4 *>(lds + 4 * kWaveFloatsB);   // CH = 2: [packet parity][pair][4][lane]

  // ---- transformed filters: source channel c of this pass is the layer's filter index, output k its
  // input channel, the taps rotated: g[r][s] = w[c][k][2 - r][2 - s]; per (channel half, output group)
  float U[4][16];
#pragma unroll
  for (int cb = 0; cb < CH * KT; ++cb) {
    const int ch = cb % CH, kt = cb / CH;
    {
      const int c = tid >> 4, k = tid & 15;
      const float *g = a.w + ((long)(16 * ch + c) * kKout + 16 * kt + k) * 9;
      float gv[9];
#pragma unroll
      for (int e = 0; e < 9; ++e) gv[e] = g[8 - e];
      float t[4][3];
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        t[0][j] = gv[j];
        t[1][j] = 0.5f * (gv[j] + gv[3 + j] + gv[6 + j]);
        t[2][j] = 0.5f * (gv[j] - gv[3 + j] + gv[6 + j]);
        t[3][j] = gv[6 + j];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        lds[((4 * i + 0) * 16 + c) * 16 + k] = t[i][0];
        lds[((4 * i + 1) * 16 + c) * 16 + k] = 0.5f * (t[i][0] + t[i][1] + t[i][2]);
        lds[((4 * i + 2) * 16 + c) * 16 + k] = 0.5f * (t[i][0] - t[i][1] + t[i][2]);
        lds[((4 * i + 3) * 16 + c) * 16 + k] = t[i][2];
      }
    }
    __syncthreads();
    if (ch == chalf && kt == ktile) {
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int q = 0; q < 16; ++q) U[s][q] = lds[(q * 16 + 4 * s + kq) * 16 + i16];
    }
    __syncthreads();
  }

  const __amdgpu_buffer_rsrc_t rs_g = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.src), 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_f = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(a.src_idx), 0, (int)(p.x_bytes >> 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, (int)p.y_bytes, 0x00020000);

  // Packet slots.  Main: (channel lane >> 2, windows 4j .. 4j+3 of the segment, j = lane & 3): 16 bytes of
  // gradient and 4 pooling bytes.  Neighbours (lanes 0 .. 31): (channel lane >> 1, the window left of the
  // segment or right of it): one gradient, one byte.
  const int m_ch = lane >> 2, m_j = lane & 3;
  const int m_lo = m_ch * kPSB + 8 * m_j + 1;             // LDS: image column x0 sits at column 1
  const int n_ch = (lane & 31) >> 1, n_side = lane & 1;
  const int n_lo = n_ch * kPSB + (n_side ? 33 : 0);
  const int plane = p.Hp * p.Wp;
  int me = 0, ne = 0;              // element offsets of the lane's slots in the first packet of the item being requested
  bool mok = false, nok = false;
  auto item_setup = [&](int n, int bx0, int by0) {
    const int base = ((n * kCin + c0) * p.Hp + (by0 - 1)) * p.Wp + bx0;
    me = base + m_ch * plane + 4 * m_j;
    mok = bx0 + 4 * m_j < p.Wp;
    const int nc = bx0 + (n_side ? 16 : -1);
    ne = base + n_ch * plane + (n_side ? 16 : -1);
    nok = lane < 32 && bx0 < p.Wp && (unsigned)nc < (unsigned)p.Wp;
  };
  struct Packet {
    float4 g;
    unsigned f;
    float ng;
    unsigned nf;
  };
  Packet pa, pb;
  pa.g = pb.g = make_float4(0.f, 0.f, 0.f, 0.f);
  pa.f = pb.f = pa.nf = pb.nf = 0;
  pa.ng = pb.ng = 0.0f;
  // pooled row R -> registers; dP = R - (by0 - 1).  A row above or below the map is asked for out of range
  auto load_packet = [&](int R, int dP, Packet &k) {
    const bool none = R < 0 || R >= p.Hp;
    const unsigned e = (unsigned)(me + p.Wp * dP), en = (unsigned)(ne + p.Wp * dP);
    const bool ok = mok && !none, okn = nok && !none;
    const floatx4 v = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rs_g, (int)(ok ? 4u * e : kOob), 0, 0));
    k.g = make_float4(v[0], v[1], v[2], v[3]);
    k.f = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(rs_f, (int)(ok ? e : kOob), 0, 0);
    k.ng = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_g, (int)(okn ? 4u * en : kOob), 0, 0));
    k.nf = (unsigned)__builtin_amdgcn_raw_buffer_load_b8(rs_f, (int)(okn ? en : kOob), 0, 0);
  };
  // registers -> the two dz rows of the packet's windows in slot pair `slot` (out-of-range loads gave
  // zeros: zero gradient, zeros written)
  auto scatter = [&](int slot, const Packet &k) {
    float *r0 = xs + slot * 2 * kRS + m_lo, *r1 = r0 + kRS;
    const float gq[4] = {k.g.x, k.g.y, k.g.z, k.g.w};
    float z0[8], z1[8];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const unsigned f = (k.f >> (8 * w)) & 0xffu;
      const float v = (f & kIdxInactive) ? 0.0f : gq[w];
      const unsigned pos = f & kIdxPosMask;
      z0[2 * w] = pos == 0 ? v : 0.0f;
      z0[2 * w + 1] = pos == 1 ? v : 0.0f;
      z1[2 * w] = pos == 2 ? v : 0.0f;
      z1[2 * w + 1] = pos == 3 ? v : 0.0f;
    }
    r0[0] = z0[0];
    *reinterpret_cast<float2 *>(r0 + 1) = make_float2(z0[1], z0[2]);
    *reinterpret_cast<float2 *>(r0 + 3) = make_float2(z0[3], z0[4]);
    *reinterpret_cast<float2 *>(r0 + 5) = make_float2(z0[5], z0[6]);
    r0[7] = z0[7];
    r1[0] = z1[0];
    *reinterpret_cast<float2 *>(r1 + 1) = make_float2(z1[1], z1[2]);
    *reinterpret_cast<float2 *>(r1 + 3) = make_float2(z1[3], z1[4]);
    *reinterpret_cast<float2 *>(r1 + 5) = make_float2(z1[5], z1[6]);
    r1[7] = z1[7];
    if (lane < 32) {
      // the left neighbour window shows its right column (positions 1, 3), the right one its left column (0, 2)
      const float v = (k.nf & kIdxInactive) ? 0.0f : k.ng;
      const unsigned pos = k.nf & kIdxPosMask, col = n_side ? 0u : 1u;
      float *d = xs + slot * 2 * kRS + n_lo;
      d[0] = pos == col ? v : 0.0f;
      d[kRS] = pos == col + 2u ? v : 0.0f;
    }
  };

  // ---- one block row: 16 blocks x 16 output channels; s0, s1, s2: slot pairs of the pooled rows by-1, by, by+1
  const float *patch = xs + kq * kPSB + 2 * i16;
  const floatx4 zero = {0.f, 0.f, 0.f, 0.f};
  // The input transform is taken row-wise first, as in the forward kernel: H = d B of a dz row serves
  // two block rows (the upper row of pooled row R as row 3 of block row R-1 and row 1 of block row R,
  // the lower one as row 2 of block row R and row 0 of block row R+1), so the H of a packet's two dz rows
  // is computed once, when the packet arrives, and kept: `X` holds the rows of the packet before last
  // and receives the arriving packet's (its upper row at once - the old one is no longer needed -, its
  // lower row after the old lower row has been used as row 0 of the block row worked now), `Y` those of
  // the packet before.  The two sets swap roles from packet to packet.
  struct HSet { float u[4][4], l[4][4]; };   // [channel quartet][value]: upper and lower dz row of a pooled row
  auto h_row = [&](const float2 &l, const float2 &h, float (&o)[4]) {
    o[0] = l.x - h.x;
    o[1] = l.y + h.x;
    o[2] = h.x - l.y;
    o[3] = l.y - h.y;
  };
  // a packet with no block row to work (the first two of an item): only its H is taken
  auto prime = [&](int slot, HSet &X) {
    const float *pnew = patch + 2 * slot * kRS;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const float *row = pnew + 4 * s * kPSB;
      h_row(*reinterpret_cast<const float2 *>(row), *reinterpret_cast<const float2 *>(row + 2), X.u[s]);
      h_row(*reinterpret_cast<const float2 *>(row + kRS), *reinterpret_cast<const float2 *>(row + kRS + 2), X.l[s]);
    }
  };
  auto block_row = [&](int slot, HSet &X, const HSet &Y, floatx4 (&z)[4]) {
    const float *pnew = patch + 2 * slot * kRS;   // the two dz rows of the packet just scattered
    floatx4 acc[16];
    float2 pl[2][2], ph[2][2];
    auto read_patch = [&](auto sc) {
      constexpr int s = decltype(sc)::value;
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        const float *row = pnew + r * kRS + 4 * s * kPSB;
        pl[s & 1][r] = *reinterpret_cast<const float2 *>(row);
        ph[s & 1][r] = *reinterpret_cast<const float2 *>(row + 2);
      }
    };
    auto quartet = [&](auto sc) {
      constexpr int s = decltype(sc)::value;
      if constexpr (s < 3) read_patch(std::integral_constant<int, s + 1>{});
      __builtin_amdgcn_sched_barrier(0);
      // V = Bt H over the rows X.l (old), Y.u, Y.l, X.u (new)
      float V[16];
#pragma unroll
      for (int j = 0; j < 4; ++j) V[j] = X.l[s][j] - Y.l[s][j];
      h_row(pl[s & 1][0], ph[s & 1][0], X.u[s]);
      h_row(pl[s & 1][1], ph[s & 1][1], X.l[s]);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        V[4 + j] = Y.u[s][j] + Y.l[s][j];
        V[8 + j] = Y.l[s][j] - Y.u[s][j];
        V[12 + j] = Y.u[s][j] - X.u[s][j];
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(V[q], U[s][q], s == 0 ? zero : acc[q], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    };
    read_patch(std::integral_constant<int, 0>{});
    quartet(std::integral_constant<int, 0>{});
    quartet(std::integral_constant<int, 1>{});
    quartet(std::integral_constant<int, 2>{});
    quartet(std::integral_constant<int, 3>{});
    // ---- output transform: z[v] = the 2x2 block 4kq+v (y00, y01, y10, y11)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      float sr[2][4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        sr[0][j] = acc[j][v] + acc[4 + j][v] + acc[8 + j][v];
        sr[1][j] = acc[4 + j][v] - acc[8 + j][v] - acc[12 + j][v];
      }
      z[v] = floatx4{sr[0][0] + sr[0][1] + sr[0][2], sr[0][1] - sr[0][2] - sr[0][3],
                     sr[1][0] + sr[1][1] + sr[1][2], sr[1][1] - sr[1][2] - sr[1][3]};
    }
  };

  auto rows_of = [&](int item, int &n_img, int &xseg, int &by0) -> int {
    const int xg = item % p.xgroups;
    const int rgrp = (item / p.xgroups) % p.rgroups;
    n_img = item / (p.xgroups * p.rgroups);
    xseg = xg * S + stream;
    by0 = rgrp * p.rg;
    return (CH == 2 || xseg < p.xsegs) ? min(by0 + p.rg, p.Hp) - by0 : 0;
  };
  int r_item = gidx - p.G, r_q = 0, r_n = -1, r_by0 = 0;
  auto next_request_item = [&]() {
    int n_img = 0, xseg = 0;
    r_n = 0;
    for (r_item += p.G; r_item < p.items; r_item += p.G)
      if ((r_n = rows_of(r_item, n_img, xseg, r_by0)) > 0) break;
    r_q = 0;
    if (r_item < p.items) {
      item_setup(n_img, xseg * 16, r_by0);
    } else {
      mok = nok = false;
      r_by0 = 0;
    }
  };
  auto request = [&](Packet &k) {
    load_packet(r_by0 - 1 + r_q, r_q, k);
    if (++r_q > r_n + 1) next_request_item();
  };
  int c_item = gidx - p.G, c_q = 0, c_n = -1, c_slot = 0, c_par = 0;
  unsigned c_yo = kOob;   // element offset of the lane's outputs in the item's first block row
  auto next_consume_item = [&]() {
    int n_img = 0, xseg = 0, by0 = 0;
    c_n = 0;
    for (c_item += p.G; c_item < p.items; c_item += p.G)
      if ((c_n = rows_of(c_item, n_img, xseg, by0)) > 0) break;
    c_q = 0;
    c_slot = 0;
    const int x = xseg * 32 + 8 * kq;
    c_yo = (c_item < p.items && x < a.Wout) ? (unsigned)(((n_img * kKout + k0 + i16) * a.Hout + 2 * by0) * a.Wout + x) : kOob;
  };
  auto handle = [&](Packet &k, HSet &X, const HSet &Y) {
    const bool live = c_item < p.items;
    scatter(c_slot, k);
    request(k);
    floatx4 z[4] = {zero, zero, zero, zero};
    unsigned yo = kOob;
    const bool work = live && c_q > 1;
    if (work) block_row(c_slot, X, Y, z);
    else prime(c_slot, X);
    if constexpr (CH == 2) {
      floatx4 *ex = exch + ((c_par * 2 + wave / 2) * 4) * 64 + lane;
      if (chalf == 1) {
#pragma unroll
        for (int v = 0; v < 4; ++v) ex[64 * v] = z[v];
      }
      __syncthreads();
      if (chalf == 0) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const floatx4 o = ex[64 * v];
          z[v] += o;
        }
      }
      c_par ^= 1;
    }
    if (work && chalf == 0 && c_yo != kOob) yo = 4u * (c_yo + (unsigned)(2 * (c_q - 2) * a.Wout));
    // the lane's blocks 4kq .. 4kq+3 are eight neighbouring columns of two rows
    const floatx4 y[4] = {floatx4{z[0][0], z[0][1], z[1][0], z[1][1]}, floatx4{z[2][0], z[2][1], z[3][0], z[3][1]},
                          floatx4{z[0][2], z[0][3], z[1][2], z[1][3]}, floatx4{z[2][2], z[2][3], z[3][2], z[3][3]}};
    const unsigned rowb = 4u * (unsigned)a.Wout;
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uintx4, y[0]), rs_y, (int)yo, 0, 0);
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uintx4, y[1]), rs_y, (int)(yo == kOob ? kOob : yo + 16u), 0, 0);
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uintx4, y[2]), rs_y, (int)(yo == kOob ? kOob : yo + rowb), 0, 0);
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uintx4, y[3]), rs_y, (int)(yo == kOob ? kOob : yo + rowb + 16u), 0, 0);
    if (live) {
      c_slot = c_slot == 2 ? 0 : c_slot + 1;
      if (++c_q > c_n + 1) next_consume_item();
    }
  };

  next_request_item();
  next_consume_item();
  auto empty_stores = [&]() {
#pragma unroll
    for (int q = 0; q < 4; ++q)   // four different (out-of-range) places: identical stores would be merged into one
      __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uintx4, zero), rs_y, (int)(kOob + 16u * (unsigned)q), 0, 0);
  };
  request(pa);
  empty_stores();
  request(pb);
  empty_stores();
  HSet HA = {}, HB = {};
  while (c_item < p.items) {
    handle(pa, HA, HB);
    handle(pb, HB, HA);
  }
}

template <int KT, int CH>
__global__ __launch_bounds__(kThreads, 2) void conv3x3_wino_stream_bwd_kernel(const WinoStreamParams p) {
  extern __shared__ float lds[];
  stream_bwd_body<KT, CH>(p, lds, blockIdx.x);
}

// A layer's filter gradient and its backward-data pass read the same gradient and do not depend on
// each other: one launch runs both, half of the workgroups each (roles alternate in groups of eight
// workgroup indices, so that each of the eight XCDs - indices go to them in turn - gets both), and the
// ramp and drain of a launch are paid once instead of twice.  Both bodies walk their work items
// with the stride of their own workgroup count, so neither knows of the other.
template <int KT, int CT>
__global__ __launch_bounds__(kThreads, 2) void wgrad_bwd_pair_kernel(const wgw::WinoWgradParams pw, const WinoStreamParams pb) {
  extern __shared__ float lds[];
  const int role = (blockIdx.x >> 3) & 1, idx = (int)(((blockIdx.x >> 4) << 3) | (blockIdx.x & 7));
  // filter gradient: K filters (KT tiles) x C channels (CT tiles); backward-data of the same layer: K source
  // channels (halves: KT) -> C outputs (groups: CT)
  if (role) wgw::wgrad_wino_body<KT, CT>(pw, lds, idx);
  else stream_bwd_body<CT, KT>(pb, lds, idx);
}

inline bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

}  // namespace

namespace {
// streams of a workgroup for a layer with `cin` source channels and `kout` outputs, or 0 when the kernels do not take it
// (32 -> 32 channels stay with the tile kernel: on config 5's 32 x 32 maps the single stream of such a
// workgroup has one short item, and the pass measured 20.9 against 18.0 us)
int stream_count(int cin, int kout, bool both32 = false) {
  if ((cin != 16 && cin != 32) || (kout != 16 && kout != 32) || (cin == 32 && kout == 32 && !both32)) return 0;
  return 4 / ((cin / 16) * (kout / 16));
}
// a 32-channel source is worked by wavefront pairs that meet at a barrier per packet: every stream of
// a workgroup must then have a segment in every item
bool streams_filled(const ConvEngineArgs &a, bool both32 = false) {
  const int S = stream_count(a.Cin, a.Kout, both32);
  return S > 0 && (a.Cin == 16 || ((a.Win + 31) / 32) % S == 0);
}

void fill_params(const ConvEngineArgs &a, WinoStreamParams &p, long workgroups = 0) {
  const int streams = stream_count(a.Cin, a.Kout, true);
  p.a = a;
  p.Hp = a.Hin / 2;
  p.Wp = a.Win / 2;
  p.xsegs = (a.Win + 31) / 32;
  p.xgroups = (p.xsegs + streams - 1) / streams;
  // two workgroups per compute unit (registers), unless the launch is shared and the caller says how many are this pass's
  const long resident = workgroups > 0 ? workgroups : 2L * chip().cus;
  // block rows per work item: long strips re-read fewer halo rows, short ones balance the workgroups;
  // the first length that leaves every resident workgroup an item, else the shortest
  p.rg = 2;
  for (int rg = 16; rg >= 2; rg /= 2) {
    const long items = (long)a.N * p.xgroups * ((p.Hp + rg - 1) / rg);
    if (items >= resident || rg == 2) { p.rg = rg; break; }
  }
  p.rgroups = (p.Hp + p.rg - 1) / p.rg;
  p.items = a.N * p.rgroups * p.xgroups;
  p.G = (int)(p.items < resident ? p.items : resident);
}

template <typename Kern>
hipError_t launch_stream(Kern kern, const WinoStreamParams &p, size_t lds_bytes, hipStream_t stream) {
  const hipError_t e = allow_large_lds(reinterpret_cast<const void *>(kern), lds_bytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(p.G), dim3(kThreads), lds_bytes, stream, p);
  return hipGetLastError();
}
constexpr size_t kExchBytes = sizeof(floatx4) * 2 * 2 * 4 * 64;   // two packet parities x two wavefront pairs x 4 x 64 lanes
}  // namespace

bool conv_wino_stream_applies(const ConvEngineArgs &a) {
  if (a.src_dz || a.w_flip || a.R != 3 || a.S != 3 || a.pad_h != 1 || a.pad_w != 1) return false;
  if (!streams_filled(a) || a.act != ACT_RELU || a.pool != 2) return false;
  if (a.Hout != a.Hin || a.Wout != a.Win || a.Win % 8 != 0 || a.Hin % 2 != 0 || a.Win >= (1 << 17)) return false;
  if (a.uniform || a.sample || a.out_pool) return false;
  if (!aligned16(a.src) || !aligned16(a.out) || (a.out_idx && (reinterpret_cast<uintptr_t>(a.out_idx) & 3u))) return false;
  const long limit = (1L << 31) - (1L << 24);
  return 4L * a.N * a.Cin * a.Hin * a.Win < limit && 4L * a.N * a.Kout * (a.Hin / 2) * (a.Win / 2) < limit;
}

namespace {
bool stream_bwd_ok(const ConvEngineArgs &a, bool both32);
}
bool conv_wino_stream_bwd_applies(const ConvEngineArgs &a) { return stream_bwd_ok(a, false); }
namespace {
bool stream_bwd_ok(const ConvEngineArgs &a, bool both32) {
  if (!a.src_dz || !a.w_flip || a.src_pool != 2 || a.src_act != ACT_RELU_FLAGGED || !a.src_idx) return false;
  if (a.R != 3 || a.S != 3 || a.pad_h != 1 || a.pad_w != 1 || !streams_filled(a, both32)) return false;
  if (a.act != ACT_IDENTITY || a.pool != 1 || a.bias || a.uniform || a.sample || a.out_pool) return false;
  if (a.Hout != a.Hin || a.Wout != a.Win || a.Win % 8 != 0 || a.Hin % 2 != 0 || a.Win >= (1 << 17)) return false;
  if (!aligned16(a.src) || !aligned16(a.out) || (reinterpret_cast<uintptr_t>(a.src_idx) & 3u)) return false;
  const long limit = (1L << 31) - (1L << 24);
  return 4L * a.N * a.Kout * a.Hin * a.Win < limit && 4L * a.N * a.Cin * (a.Hin / 2) * (a.Win / 2) < limit;
}
}  // namespace

hipError_t launch_conv_wino_stream(const ConvEngineArgs &a, hipStream_t stream) {
  static_assert(4 * kWaveFloats >= 16 * 16 * 16 && 4 * kWaveFloatsB >= 16 * 16 * 16, "the transformed filters pass through the rings' memory");
  WinoStreamParams p;
  const int KT = a.Kout / 16, CH = a.Cin / 16;
  if (conv_wino_stream_bwd_applies(a)) {
    fill_params(a, p);
    p.x_bytes = (unsigned)(4L * a.N * a.Cin * p.Hp * p.Wp);
    p.y_bytes = (unsigned)(4L * a.N * a.Kout * a.Hin * a.Win);
    const size_t lds = sizeof(float) * 4 * kWaveFloatsB + (CH == 2 ? kExchBytes : 0);
    if (KT == 1 && CH == 1) return launch_stream(conv3x3_wino_stream_bwd_kernel<1, 1>, p, lds, stream);
    if (KT == 2 && CH == 1) return launch_stream(conv3x3_wino_stream_bwd_kernel<2, 1>, p, lds, stream);
    return launch_stream(conv3x3_wino_stream_bwd_kernel<1, 2>, p, lds, stream);
  }
  if (!conv_wino_stream_applies(a)) return hipErrorInvalidValue;
  fill_params(a, p);
  p.x_bytes = (unsigned)(4L * a.N * a.Cin * a.Hin * a.Win);
  p.y_bytes = (unsigned)(4L * a.N * a.Kout * p.Hp * p.Wp);
  const size_t lds = sizeof(float) * 4 * kWaveFloats + (CH == 2 ? kExchBytes : 0);
  if (a.out_idx) {
    if (KT == 1 && CH == 1) return launch_stream(conv3x3_wino_stream_kernel<true, 1, 1>, p, lds, stream);
    if (KT == 2 && CH == 1) return launch_stream(conv3x3_wino_stream_kernel<true, 2, 1>, p, lds, stream);
    return launch_stream(conv3x3_wino_stream_kernel<true, 1, 2>, p, lds, stream);
  }
  if (KT == 1 && CH == 1) return launch_stream(conv3x3_wino_stream_kernel<false, 1, 1>, p, lds, stream);
  if (KT == 2 && CH == 1) return launch_stream(conv3x3_wino_stream_kernel<false, 2, 1>, p, lds, stream);
  return launch_stream(conv3x3_wino_stream_kernel<false, 1, 2>, p, lds, stream);
}

// The filter gradient (plan with `cus` workgroups) and the backward-data pass of one layer in one launch.
bool wgrad_bwd_pair_applies(const WgradArgs &w, const WgradPlan &plan, const ConvEngineArgs &b) {
  // (in a shared launch the streaming backward-data form also takes 32 -> 32 channels: on its own it is
  // slower than the tile kernel there, but less so than a launch costs)
  if (!wgrad_wino_applies(w, plan) || !stream_bwd_ok(b, true)) return false;
  if (w.C == 32 && w.K != 32) return false;          // 32 -> 16 channels: its backward-data pass (16 -> 32) has a form, its pair is not built
  if (b.Cin != w.K || b.Kout != w.C || b.N != w.N || b.Hin != w.H || b.Win != w.W) return false;
  WinoStreamParams pb;
  fill_params(b, pb, plan.G);
  return pb.G == plan.G && plan.G % 8 == 0;          // equal halves, whole groups of eight
}

hipError_t launch_wgrad_bwd_pair(const WgradArgs &w, const WgradPlan &plan, const ConvEngineArgs &b, hipStream_t stream) {
  if (!wgrad_bwd_pair_applies(w, plan, b)) return hipErrorInvalidValue;
  wgw::WinoWgradParams pw;
  if (!wgw::fill_wino_wgrad_params(w, plan, pw)) return hipErrorInvalidValue;
  WinoStreamParams pb;
  fill_params(b, pb, plan.G);
  pb.x_bytes = (unsigned)(4L * b.N * b.Cin * pb.Hp * pb.Wp);
  pb.y_bytes = (unsigned)(4L * b.N * b.Kout * b.Hin * b.Win);
  const int KT = w.K / 16, CT = w.C / 16;
  size_t lds = sizeof(float) * 4 * kWaveFloatsB + (KT == 2 ? kExchBytes : 0);
  if (lds < wgw::kWinoWgradLdsBytes) lds = wgw::kWinoWgradLdsBytes;
  const dim3 grid((unsigned)(2 * plan.G)), block(kThreads);
  hipError_t e;
  if (KT == 1) {
    if ((e = allow_large_lds(reinterpret_cast<const void *>(wgrad_bwd_pair_kernel<1, 1>), lds)) != hipSuccess) return e;
    hipLaunchKernelGGL((wgrad_bwd_pair_kernel<1, 1>), grid, block, lds, stream, pw, pb);
  } else if (CT == 2) {
    if ((e = allow_large_lds(reinterpret_cast<const void *>(wgrad_bwd_pair_kernel<2, 2>), lds)) != hipSuccess) return e;
    hipLaunchKernelGGL((wgrad_bwd_pair_kernel<2, 2>), grid, block, lds, stream, pw, pb);
  } else {
    if ((e = allow_large_lds(reinterpret_cast<const void *>(wgrad_bwd_pair_kernel<2, 1>), lds)) != hipSuccess) return e;
    hipLaunchKernelGGL((wgrad_bwd_pair_kernel<2, 1>), grid, block, lds, stream, pw, pb);
  }
  return hipGetLastError();
}

}  // namespace dllk
