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
  int xsegs, xgroups;  // 32-pixel column segments; groups of four neighbouring segments (one per wavefront)
  int rg, rgroups;     // block rows per work item, row groups per image
  int items;           // work items of a workgroup: N * rgroups * xgroups
  int G;               // workgroups
  unsigned x_bytes, y_bytes;
};

template <bool IDX>
__global__ __launch_bounds__(kThreads, 2) void conv3x3_wino_stream_kernel(const WinoStreamParams p) {
  extern __shared__ float lds[];
  const ConvEngineArgs &a = p.a;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same in every lane: it lives in scalar registers
  const int i16 = lane & 15, kq = lane >> 4;
  const int gidx = blockIdx.x;
  float *xs = lds + wave * kWaveFloats;

  // ---- transformed filters U = G g Gt, G = [1 0 0; .5 .5 .5; .5 -.5 .5; 0 0 1]: one (channel, filter)
  // pair per thread into LDS [point][channel][filter] (over the rings, which are not in use yet), then
  // each lane takes its B fragments: channel 4s+kq, filter i16, every point
  {
    const int c = tid >> 4, k = tid & 15;
    const float *g = a.w + ((long)k * 16 + c) * 9;
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
  float U[4][16];
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int q = 0; q < 16; ++q) U[s][q] = lds[(q * 16 + 4 * s + kq) * 16 + i16];
  __syncthreads();   // everybody has its fragments: the rings may be written
  const float bias = a.bias ? a.bias[i16] : 0.0f;

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
    const int base = ((n * 16) * a.Hin + (2 * by0 - 1)) * a.Win + x0;
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
  auto block_row = [&](int sp, floatx4 &y, unsigned &ib) {
    const float *pup = patch + sp * 2 * kRS, *pdn = patch + (sp ^ 1) * 2 * kRS;
    floatx4 acc[16];
    float2 pl[2][4], ph[2][4];
    auto read_patch = [&](auto sc) {
      constexpr int s = decltype(sc)::value;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float *row = (i < 2 ? pup + i * kRS : pdn + (i - 2) * kRS) + 4 * s * kPS;
        pl[s & 1][i] = *reinterpret_cast<const float2 *>(row);
        ph[s & 1][i] = *reinterpret_cast<const float2 *>(row + 2);
      }
    };
    auto quartet = [&](auto sc) {
      constexpr int s = decltype(sc)::value;
      if constexpr (s < 3) read_patch(std::integral_constant<int, s + 1>{});
      __builtin_amdgcn_sched_barrier(0);
      // ---- V = Bt d B, Bt = [1 0 -1 0; 0 1 1 0; 0 -1 1 0; 0 1 0 -1]
      float t[4][4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float d0 = j < 2 ? (j ? pl[s & 1][0].y : pl[s & 1][0].x) : (j == 2 ? ph[s & 1][0].x : ph[s & 1][0].y);
        const float d1 = j < 2 ? (j ? pl[s & 1][1].y : pl[s & 1][1].x) : (j == 2 ? ph[s & 1][1].x : ph[s & 1][1].y);
        const float d2 = j < 2 ? (j ? pl[s & 1][2].y : pl[s & 1][2].x) : (j == 2 ? ph[s & 1][2].x : ph[s & 1][2].y);
        const float d3 = j < 2 ? (j ? pl[s & 1][3].y : pl[s & 1][3].x) : (j == 2 ? ph[s & 1][3].x : ph[s & 1][3].y);
        t[0][j] = d0 - d2;
        t[1][j] = d1 + d2;
        t[2][j] = d2 - d1;
        t[3][j] = d1 - d3;
      }
      float V[16];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        V[4 * i + 0] = t[i][0] - t[i][2];
        V[4 * i + 1] = t[i][1] + t[i][2];
        V[4 * i + 2] = t[i][2] - t[i][1];
        V[4 * i + 3] = t[i][1] - t[i][3];
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
    // ---- output transform At M A, At = [1 1 1 0; 0 1 -1 -1], then bias, ReLU, pooling: a block is one window
    float yv[4];
    ib = 0;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      float sr[2][4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        sr[0][j] = acc[j][v] + acc[4 + j][v] + acc[8 + j][v];
        sr[1][j] = acc[4 + j][v] - acc[8 + j][v] - acc[12 + j][v];
      }
      const float y00 = sr[0][0] + sr[0][1] + sr[0][2], y01 = sr[0][1] - sr[0][2] - sr[0][3];
      const float y10 = sr[1][0] + sr[1][1] + sr[1][2], y11 = sr[1][1] - sr[1][2] - sr[1][3];
      float m = y00;
      unsigned arg = 0;
      if (y01 > m) { m = y01; arg = 1; }
      if (y10 > m) { m = y10; arg = 2; }
      if (y11 > m) { m = y11; arg = 3; }
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
    xseg = xg * 4 + wave;
    by0 = rgrp * p.rg;
    return xseg < p.xsegs ? min(by0 + p.rg, p.Hp) - by0 : 0;
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
  int c_item = gidx - p.G, c_q = 0, c_n = -1;
  unsigned c_yo = kOob;   // element offset of the lane's outputs in the item's first block row
  auto next_consume_item = [&]() {
    int n_img = 0, xseg = 0, by0 = 0;
    c_n = 0;
    for (c_item += p.G; c_item < p.items; c_item += p.G)
      if ((c_n = rows_of(c_item, n_img, xseg, by0)) > 0) break;
    c_q = 0;
    const int bx = xseg * 16 + 4 * kq;
    c_yo = (c_item < p.items && bx < p.Wp) ? (unsigned)(((n_img * 16 + i16) * p.Hp + by0) * p.Wp + bx) : kOob;
  };
  // (a packet handled after the wavefront's last item is an empty one: the loop below leaves only after
  // whole rounds of both register sets, so that no path leads from one set's packet straight to the
  // same set's next - the compiler would have to assume the loads just issued are the ones awaited)
  auto handle = [&](float4 (&xr)[kXR], float &xh) {
    const bool live = c_item < p.items;
    store_pair(c_q & 1, xr, xh);
    request(xr, xh);
    // the stores are issued for every packet (out of range where no block row was worked), like the loads
    floatx4 y = zero;
    unsigned ib = 0, yo = kOob;
    if (live && c_q > 0) {
      block_row((c_q - 1) & 1, y, ib);
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
  while (c_item < p.items) {
    handle(xa, ha);
    handle(xb, hb);
  }
}

inline bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

}  // namespace

bool conv_wino_stream_applies(const ConvEngineArgs &a) {
  if (a.src_dz || a.w_flip || a.R != 3 || a.S != 3 || a.pad_h != 1 || a.pad_w != 1) return false;
  if (a.Cin != 16 || a.Kout != 16 || a.act != ACT_RELU || a.pool != 2) return false;
  if (a.Hout != a.Hin || a.Wout != a.Win || a.Win % 8 != 0 || a.Hin % 2 != 0 || a.Win >= (1 << 17)) return false;
  if (a.uniform || a.sample || a.out_pool) return false;
  if (!aligned16(a.src) || !aligned16(a.out) || (a.out_idx && (reinterpret_cast<uintptr_t>(a.out_idx) & 3u))) return false;
  const long limit = (1L << 31) - (1L << 24);
  return 4L * a.N * a.Cin * a.Hin * a.Win < limit && 4L * a.N * a.Kout * (a.Hin / 2) * (a.Win / 2) < limit;
}

hipError_t launch_conv_wino_stream(const ConvEngineArgs &a, hipStream_t stream) {
  if (!conv_wino_stream_applies(a)) return hipErrorInvalidValue;
  WinoStreamParams p;
  p.a = a;
  p.Hp = a.Hin / 2;
  p.Wp = a.Win / 2;
  p.xsegs = (a.Win + 31) / 32;
  p.xgroups = (p.xsegs + 3) / 4;
  p.x_bytes = (unsigned)(4L * a.N * a.Cin * a.Hin * a.Win);
  p.y_bytes = (unsigned)(4L * a.N * a.Kout * p.Hp * p.Wp);
  const long resident = 2L * chip().cus;   // two workgroups per compute unit (registers)
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
  const size_t smem = sizeof(float) * 4 * kWaveFloats;
  static_assert(4 * kWaveFloats >= 16 * 16 * 16, "the transformed filters pass through the rings' memory");
  if (a.out_idx) hipLaunchKernelGGL(conv3x3_wino_stream_kernel<true>, dim3(p.G), dim3(kThreads), smem, stream, p);
  else hipLaunchKernelGGL(conv3x3_wino_stream_kernel<false>, dim3(p.G), dim3(kThreads), smem, stream, p);
  return hipGetLastError();
}

}  // namespace dllk
