// Filter gradient of the padded 3x3 layers with 16 or 32 channels in and out behind ReLU + 2x2 max
// pooling, in the minimal-filtering form F(3x3, 2x2), on fp32 MFMA (v_mfma_f32_16x16x4_f32), gfx950.
//
//   dw[k,c,r,s] = sum_{n,i,j} dz[n,k,i,j] * xpad[n,c,i+r,j+s]      (Section II-A, gradient computations)
//
// Seen per 2x2 block of dz, the nine sums are a 3x3-output correlation of the block (the "filter")
// with the 4x4 patch of x around it:  dw = sum_blocks A^T [ (G g G^T) .* (B^T d B) ] A  with
//   B^T = [1 0 -1 0; 0 1 1 0; 0 -1 1 0; 0 1 0 -1],  G = [1 0; 1 1; 1 -1; 0 -1],  A^T = [1 .5 .5 0; 0 .5 -.5 0; 0 .5 .5 1]
// (the transposed form of the F(2x2, 3x3) matrices the forward kernel uses).  The sums over blocks
// and images of the 16 point-wise products are the matrix part: per transform point p,
// M_p[k][c] = sum_blocks U_p[k][block] * V_p[c][block], 16 x 16 x 4 blocks per MFMA: four
// instructions per block of four pixels where the direct sum takes nine; A^T . A is applied once,
// at the very end.  The pooled layer makes the filter-side transform trivial: a 2x2 block of dz is
// one pooling window and holds at most one non-zero, dy at the recorded position (a, b), so
// U = dy * (G[:,a] outer G[:,b]) has entries 0 and +-dy only: selects, no arithmetic.
//
// Layout: filters on the MFMA M axis, channels on N, blocks on K.  Lane (i16, kq) builds U for
// filter i16 and V for channel i16 of ITS block, register-local: the x patch comes from LDS as four
// rows of two 8-byte reads, dy and the pooling byte straight from global memory (16 consecutive
// blocks of a filter row are four lanes' 16-byte loads).  Every wavefront works alone: its own
// (filter tile, channel tile) pair, its own strip of blocks, its own four-row ring of x rows in
// LDS (two new rows per block row, requested two block rows ahead), no workgroup barrier until the
// final, fixed-order sum of the wavefronts' results.  The partial blocks have the layout of the
// direct kernel's, so the same reduction kernel finishes both.
#pragma once
#include "dll_internal.h"

#include <type_traits>

namespace dllk {
namespace wgw {   // names of its own: the streaming forward / backward-data kernels use the same constants' names

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kRS = 36;                 // LDS row: image columns x0-1 .. x0+32 at LDS columns 0 .. 33
constexpr int kPS = 4 * kRS + 2;        // channel plane of four row slots; half of it odd: conflict-free 8-byte reads
constexpr int kWaveFloats = 16 * kPS;   // one wavefront's ring: 16 channels
constexpr int kXR = 4;                  // 16 channels x 2 rows x 8 aligned 16-byte groups = 4 per lane
constexpr unsigned kOob = 0x80000000u;

struct WinoWgradParams {
  WgradArgs a;
  int Hp, Wp;          // pooled map = blocks per column / row
  int xsegs, xgroups;  // 32-pixel column segments; groups of as many neighbouring segments as a workgroup has streams
  int rg, rgroups;     // block rows per work item, row groups per image
  int items;           // work items of a workgroup: N * rgroups * xgroups
  int G;               // workgroups = partial blocks per channel chunk
  long db_offset;
  unsigned x_bytes, dy_bytes;
};

// KT, CT: 16-filter and 16-channel tiles (1 or 2 each); the 4 / (KT * CT) remaining wavefronts of a
// workgroup are independent streams over the work items.
// (the kernel's body as a function of the workgroup's index `gidx` among p.G workgroups and its dynamic
// LDS, so that it can also run as one role of a launch that it shares with another pass)
template <int KT, int CT>
__device__ __forceinline__ void wgrad_wino_body(const WinoWgradParams &p, float *lds, const int gidx) {
  constexpr int NC = KT * CT, S = 4 / NC;
  const WgradArgs &a = p.a;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same in every lane: said so, it lives in scalar registers
  const int i16 = lane & 15, kq = lane >> 4;
  const int combo = wave % NC, stream = wave / NC;
  const int ktile = combo % KT, ctile = combo / KT;
  const int c0 = ctile * 16, k0 = ktile * 16;
  float *xs = lds + wave * kWaveFloats;

  const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.x), 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_dy = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.dy), 0, (int)p.dy_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_idx = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(a.idx), 0, (int)(p.dy_bytes >> 2), 0x00020000);

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
    xpl[it] = (ch * a.H + rr) * a.W + 4 * j;      // elements from (n, c0, first row of the pair, x0)
    xcol[it] = 4 * j;
    xlo[it] = ch * kPS + rr * kRS + 4 * j + 1;
  }
  const int h_ch = lane >> 2, h_rr = (lane >> 1) & 1, h_side = lane & 1;
  const int hpl = (h_ch * a.H + h_rr) * a.W + (h_side ? 32 : -1);
  const int hlo = h_ch * kPS + h_rr * kRS + (h_side ? 33 : 0);

  floatx4 acc[16];
#pragma unroll
  for (int q = 0; q < 16; ++q) acc[q] = floatx4{0.f, 0.f, 0.f, 0.f};
  float dbsum = 0.0f;

  float4 xa[kXR], xb[kXR];   // two pairs of rows on their way from memory to LDS
  float ha = 0.0f, hb = 0.0f;
  float4 dyc = make_float4(0.f, 0.f, 0.f, 0.f), dya = dyc, dyb = dyc;   // gradients: in use / on their way with xa / xb
  unsigned idc = 0, ida = 0, idb = 0;
  unsigned xv[kXR], hv = kOob, dv = kOob, iv = kOob;   // per-item byte offsets of the lane's slots

  // per item: where the lane's slots of the item's first pair (rows 2*by0-1, 2*by0) and first block row lie
  auto item_setup = [&](int n, int x0, int bx0, int by0) {
    const int base = ((n * a.C + c0) * a.H + (2 * by0 - 1)) * a.W + x0;
#pragma unroll
    for (int it = 0; it < kXR; ++it) xv[it] = x0 + xcol[it] < a.W ? 4u * (unsigned)(base + xpl[it]) : kOob;
    const int hc = x0 + (h_side ? 32 : -1);
    hv = (x0 < a.W && (unsigned)hc < (unsigned)a.W) ? 4u * (unsigned)(base + hpl) : kOob;
    const bool ok = bx0 + 4 * kq < p.Wp;
    const unsigned e = (unsigned)(((n * a.K + k0 + i16) * p.Hp + by0) * p.Wp + bx0 + 4 * kq);
    dv = ok ? 4u * e : kOob;
    iv = ok ? e : kOob;
  };
  // rows 2P-1 and 2P -> registers; dP = P - by0 of the item.  The pair's distance from the item's
  // first pair is added to the lanes' offsets, not passed as the loads' scalar offset: row -1 of the
  // tensor's very first plane has a negative offset, and the range check of a buffer load looks at
  // the vector offset on its own, so a negative one made good by a scalar offset would read zero.
  auto load_pair = [&](int P, int dP, float4 (&xr)[kXR], float &xh) {
    const unsigned down = (unsigned)(8 * a.W) * (unsigned)dP;
    const bool top = P == 0, bot = 2 * P >= a.H;        // the pair's first row is above / its second row below the image
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
  // pooled gradients and pooling bytes of block row by0 + dB: the lane's filter, blocks bx0 + 4kq .. + 3
  // (`none`: no such block row - the loads are issued all the same, out of range, and return zeros)
  auto load_dy = [&](int dB, bool none, float4 &g, unsigned &f) {
    const unsigned od = none ? kOob : dv, oi = none ? kOob : iv;
    const floatx4 v = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rs_dy, (int)od, (int)(4u * (unsigned)p.Wp * (unsigned)dB), 0));
    g = make_float4(v[0], v[1], v[2], v[3]);
    f = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(rs_idx, (int)oi, (int)((unsigned)p.Wp * (unsigned)dB), 0);
  };

  // one block row: four groups of four blocks; `sp` = parity of the block row inside its item = which
  // row slots hold its upper pair of rows (the lower pair sits in the other two)
  const float *patch = xs + i16 * kPS + 8 * kq;
  // The input transform V = Bt d B is taken row-wise first: H = d B for each image row (four values per
  // row, block and lane), then V = Bt H down the four rows of a patch.  Patches of neighbouring block rows
  // share two rows and the stream walks downwards, so the H of a packet's two rows is computed once, when
  // the packet arrives (`Hn`): it is the lower half of the block row worked then and, kept in registers
  // (`Hp` of the next packet), the upper half of the next one.  24 instead of 32 additions and two
  // instead of four row reads per patch; the two H sets swap roles from packet to packet.
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
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        const float *row = pnew + r * kRS + 2 * g;
        h_row(*reinterpret_cast<const float2 *>(row), *reinterpret_cast<const float2 *>(row + 2), Hn[g][r]);
      }
  };
  auto block_row = [&](int slot, const float (&Hp)[4][2][4], float (&Hn)[4][2][4]) {
    const float *pnew = patch + slot * 2 * kRS;   // the packet just stored: the block row's lower pair of rows
    const float gv[4] = {dyc.x, dyc.y, dyc.z, dyc.w};
    // the two new rows of the x patch of the lane's block of group g (rows 2by+1, 2by+2, columns
    // 2bx-1 .. 2bx+2); the reads of group g+1 are issued before the products of group g
    float2 pl[2][2], ph[2][2];
    auto read_patch = [&](auto gc) {
      constexpr int g = decltype(gc)::value;
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        const float *row = pnew + r * kRS;
        pl[g & 1][r] = *reinterpret_cast<const float2 *>(row + 2 * g);
        ph[g & 1][r] = *reinterpret_cast<const float2 *>(row + 2 * g + 2);
      }
    };
    auto group = [&](auto gc) {
      constexpr int g = decltype(gc)::value;
      if constexpr (g < 3) read_patch(std::integral_constant<int, g + 1>{});
      __builtin_amdgcn_sched_barrier(0);
      // ---- U = dy * (G[:,a] outer G[:,b]): G[:,0] = (1, 1, 1, 0), G[:,1] = (0, 1, -1, -1)
      const unsigned f = (idc >> (8 * g)) & 0xffu;
      const float v = (f & kIdxInactive) ? 0.0f : gv[g];
      if (CT == 1 || ctile == 0) dbsum += v;
      const bool pa = (f & 2u) != 0, pb = (f & 1u) != 0;
      const float R[4] = {pa ? 0.0f : v, v, pa ? -v : v, pa ? -v : 0.0f};
      // ---- V = B^T H, rows Hp[0], Hp[1], Hn[0], Hn[1]
      h_row(pl[g & 1][0], ph[g & 1][0], Hn[g][0]);
      h_row(pl[g & 1][1], ph[g & 1][1], Hn[g][1]);
      // all 32 operands first, then the 16 products back to back: a switch between the vector and the
      // matrix instruction streams costs about eight cycles each time (a loop of MFMAs with V vector
      // instructions between every two takes 33 + 8 + 4V cycles per MFMA, the same work in blocks of
      // 16 takes 33 + 4V), and left to itself the compiler alternates them
      float U[16], V[16];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        V[j] = Hp[g][0][j] - Hn[g][0][j];
        V[4 + j] = Hp[g][1][j] + Hn[g][0][j];
        V[8 + j] = Hn[g][0][j] - Hp[g][1][j];
        V[12 + j] = Hp[g][1][j] - Hn[g][1][j];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        U[4 * i + 0] = pb ? 0.0f : R[i];
        U[4 * i + 1] = R[i];
        U[4 * i + 2] = pb ? -R[i] : R[i];
        U[4 * i + 3] = pb ? -R[i] : 0.0f;
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[q] = __builtin_amdgcn_mfma_f32_16x16x4f32(U[q], V[q], acc[q], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    };
    read_patch(std::integral_constant<int, 0>{});
    group(std::integral_constant<int, 0>{});
    group(std::integral_constant<int, 1>{});
    group(std::integral_constant<int, 2>{});
    group(std::integral_constant<int, 3>{});
  };

  // ---- work items: (image, group of block rows, group of S neighbouring column segments), one segment
  // per stream, so that the wavefronts of a workgroup read neighbouring pieces of the same image
  // rows at about the same time; each stream walks its segment downwards.  A stream whose segment
  // lies beyond the row (the last group of a row that is not a multiple of S segments wide) skips
  // the item.
  //
  // The stream's work is one sequence of PACKETS: packet q of an item of n block rows (q = 0 .. n)
  // is the pair of image rows 2(by0+q)-1, 2(by0+q) together with the gradients of block row q-1
  // (none for q = 0).  Packets travel through two register sets in turn (xa/ha/dya/ida, xb/hb/dyb/idb)
  // and are requested TWO packets ahead of their use, straight across item boundaries: handling a
  // packet means moving its rows into the ring (pair q into row slots 2(q&1), 2(q&1)+1), taking its
  // gradients, asking for the packet after next into the set just emptied, and (q >= 1) multiplying
  // block row q-1, whose other pair of rows the packet before brought.  Every packet issues the same
  // seven loads on every path (when the items have run out, or for the gradients of q = 0, from
  // out-of-range offsets), so the number of loads issued after any given one is known at compile time
  // and the wait before a set is used leaves the other set's loads in flight.
  auto take = [](auto &d, auto v) { asm volatile("v_mov_b32 %0, %1" : "=v"(d) : "v"(v)); };
  auto rows_of = [&](int item, int &n_img, int &xseg, int &by0) -> int {
    const int xg = item % p.xgroups;
    const int rgrp = (item / p.xgroups) % p.rgroups;
    n_img = item / (p.xgroups * p.rgroups);
    xseg = xg * S + stream;
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
      item_setup(n_img, xseg * 32, xseg * 16, r_by0);
    } else {                                      // nothing left: every further request reads zeros
#pragma unroll
      for (int it = 0; it < kXR; ++it) xv[it] = kOob;
      hv = dv = iv = kOob;
      r_by0 = 0;
    }
  };
  auto request = [&](float4 (&xr)[kXR], float &xh, float4 &g, unsigned &f) {
    load_pair(r_by0 + r_q, r_q, xr, xh);
    load_dy(r_q > 0 ? r_q - 1 : 0, r_q == 0, g, f);
    if (++r_q > r_n) next_request_item();
  };
  int c_item = gidx - p.G, c_q = 0, c_n = -1;
  auto next_consume_item = [&]() {
    int n_img, xseg, by0;
    c_n = 0;
    for (c_item += p.G; c_item < p.items; c_item += p.G)
      if ((c_n = rows_of(c_item, n_img, xseg, by0)) > 0) break;
    c_q = 0;
  };
  // (a packet handled after the stream's last item is an empty one: the loop below leaves only after
  // whole rounds of both register sets, so that no path leads from one set's packet straight to the
  // same set's next - the compiler would have to assume the loads just issued are the ones awaited)
  auto handle = [&](float4 (&xr)[kXR], float &xh, float4 &g, unsigned &f, const float (&Hp)[4][2][4], float (&Hn)[4][2][4]) {
    const bool live = c_item < p.items;
    store_pair(c_q & 1, xr, xh);
    // real moves, here, where the packet has arrived: left to itself the compiler keeps the gradients
    // where they were loaded and moves the NEXT packet's into place at the end of the loop body
    // instead, which waits for loads that were only just issued
    take(dyc.x, g.x); take(dyc.y, g.y); take(dyc.z, g.z); take(dyc.w, g.w);
    take(idc, f);
    request(xr, xh, g, f);
    if (live && c_q > 0) block_row(c_q & 1, Hp, Hn);
    else prime(c_q & 1, Hn);
    if (live && ++c_q > c_n) next_consume_item();
  };

  next_request_item();
  next_consume_item();
  request(xa, ha, dya, ida);
  request(xb, hb, dyb, idb);
  float H0[4][2][4] = {}, H1[4][2][4] = {};
  while (c_item < p.items) {
    handle(xa, ha, dya, ida, H0, H1);
    handle(xb, hb, dyb, idb, H1, H0);
  }

  // ---- output transform, register-local: the lane holds all 16 points of filters 4kq+v, channel i16
  float out[4][9];
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    float t[3][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float m0 = acc[j][v], m1 = acc[4 + j][v], m2 = acc[8 + j][v], m3 = acc[12 + j][v];
      t[0][j] = m0 + 0.5f * (m1 + m2);
      t[1][j] = 0.5f * (m1 - m2);
      t[2][j] = 0.5f * (m1 + m2) + m3;
    }
#pragma unroll
    for (int r = 0; r < 3; ++r) {
      out[v][3 * r + 0] = t[r][0] + 0.5f * (t[r][1] + t[r][2]);
      out[v][3 * r + 1] = 0.5f * (t[r][1] - t[r][2]);
      out[v][3 * r + 2] = 0.5f * (t[r][1] + t[r][2]) + t[r][3];
    }
  }

  // ---- every wavefront drops its 16 x 16 x 9 results into LDS at their place in the partial block's
  // layout [tap tile][v][lane] (element (filter 4kq'+v, tap = channel * 9 + rs) sits at lane
  // 16kq' + tap % 16 of tap tile tap / 16); then the whole workgroup adds the streams of each
  // (filter tile, channel tile) pair in stream order and writes the block with 16-byte stores
  constexpr int SUB = 9 * 256;                     // floats of one pair's part of a partial block
  float *blk = lds;                                // [wavefront][SUB], over the wavefronts' rings
  float *dbs = lds + 4 * kWaveFloats;              // [S][KT][16]
  __syncthreads();                                 // every wavefront is done with its ring
#pragma unroll
  for (int v = 0; v < 4; ++v)
#pragma unroll
    for (int q = 0; q < 9; ++q) {
      const int tap = i16 * 9 + q;
      blk[wave * SUB + ((tap >> 4) * 4 + v) * 64 + kq * 16 + (tap & 15)] = out[v][q];
    }
  {
    float s = dbsum;
    s += __shfl_xor(s, 16, 64);
    s += __shfl_xor(s, 32, 64);
    if (kq == 0 && ctile == 0) dbs[(stream * KT + ktile) * 16 + i16] = s;
  }
  __syncthreads();
  constexpr int BLK = KT * SUB;                    // the partial block of one channel chunk: [filter tile][tap tile][v][lane]
  for (int f = tid; f < NC * (SUB / 4); f += kThreads) {
    const int cb = f / (SUB / 4), within = f - cb * (SUB / 4);
    float4 sum = *reinterpret_cast<const float4 *>(blk + cb * SUB + 4 * within);
#pragma unroll
    for (int s2 = 1; s2 < S; ++s2) {
      const float4 o = *reinterpret_cast<const float4 *>(blk + (s2 * NC + cb) * SUB + 4 * within);
      sum.x += o.x; sum.y += o.y; sum.z += o.z; sum.w += o.w;
    }
    const int kt = cb % KT, ct = cb / KT;
    *reinterpret_cast<float4 *>(a.partial + (long)(ct * p.G + gidx) * BLK + kt * SUB + 4 * within) = sum;
  }
  if (tid < KT * 16) {
    float s = dbs[tid];
#pragma unroll
    for (int s2 = 1; s2 < S; ++s2) s += dbs[s2 * KT * 16 + tid];
    a.partial[p.db_offset + (long)gidx * a.K + tid] = s;
  }
}


// host side: the launch parameters of a layer whose plan gives G workgroups
inline bool fill_wino_wgrad_params(const WgradArgs &a, const WgradPlan &plan, WinoWgradParams &p) {
  p.a = a;
  p.Hp = a.H / 2;
  p.Wp = a.W / 2;
  p.xsegs = (a.W + 31) / 32;
  p.G = plan.G;
  p.db_offset = (long)plan.db_offset;
  p.x_bytes = (unsigned)(4L * a.N * a.C * a.H * a.W);
  p.dy_bytes = (unsigned)(4L * a.N * a.K * p.Hp * p.Wp);
  const int KT = a.K / 16, CT = a.C / 16, streams = 4 / (KT * CT);
  p.xgroups = (p.xsegs + streams - 1) / streams;
  // block rows per work item: long strips re-read fewer halo rows, short ones balance the workgroups;
  // the first length that leaves every workgroup an item, else the shortest
  p.rg = 2;
  for (int rg = 8; rg >= 2; rg /= 2) {
    const long items = (long)a.N * p.xgroups * ((p.Hp + rg - 1) / rg);
    if (items >= p.G || rg == 2) { p.rg = rg; break; }
  }
  p.rgroups = (p.Hp + p.rg - 1) / p.rg;
  const long items = (long)a.N * p.xgroups * p.rgroups;
  if (items > 0x7fffffffL) return false;
  p.items = (int)items;
  return true;
}
constexpr size_t kWinoWgradLdsBytes = sizeof(float) * (4 * kWaveFloats + 4 * 2 * 16);

}  // namespace wgw
}  // namespace dllk
