// Filter gradient of a convolution layer on fp32 MFMA (v_mfma_f32_16x16x4_f32), gfx950.
//
//   dw[k,c,r,s] = sum_{n,i,j} dz[n,k,i,j] * xpad[n,c,i+r,j+s],   db[k] = sum_{n,i,j} dz[n,k,i,j]
//
// The contraction runs over pixels, so pixels sit on the MFMA K axis (4 neighbouring
// columns per instruction), filters on M and the (channel, tap) pairs of a channel chunk on
// N.  A persistent workgroup walks over image tiles of 32 x 8 output pixels: it stages the
// halo tile of x and the tile of dz = unpool(dy) * act'(y) (formed on the fly from the
// pooled-resolution tensors, never stored in HBM) in LDS and keeps its K x taps partial sums
// in accumulator registers across all its tiles.  In the fast path the next tile's global
// loads (16-byte vectors) are issued into registers before the MFMA loop of the current
// tile, so HBM latency hides behind the matrix pipe.  The four wavefronts add their
// accumulators through LDS in a fixed order and write one partial block per workgroup; a
// second kernel adds the blocks in a fixed order (no float atomics: results are
// bit-identical from run to run) and can apply the parameter update in the same pass.
#include "dll_internal.h"
#include "small_bodies.h"

#include <type_traits>

namespace dllk {

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;
constexpr int kTileW = 32;
constexpr int TH = 8;
constexpr int PSZ = TH * kTileW + 18;  // dz plane stride in LDS: half of it is odd, so A-operand reads are conflict-free
constexpr int NXI = 5;                 // prefetch registers: float4 of tile interior per thread
constexpr int NXH = 2;                 // prefetch registers: halo scalars per thread

// Offset of row r inside a dz plane.  The staging stores are 8 bytes wide and LDS serves them 16
// lanes at a time, so those 16 lanes must land in 32 different banks.  Pooled staging: 16 lanes
// hold 4 window rows x 4 column groups of 8, so window rows are 66 floats apart (2 banks) with
// the window's second row 32 floats after the first.  Unpooled staging: 16 lanes hold 2 rows x 8
// column groups of 4, so rows are 34 floats apart.
template <int POOL>
__device__ constexpr int dz_row(int r) { return POOL == 2 ? (r >> 1) * 66 + (r & 1) * kTileW : r * 34; }
static_assert(dz_row<2>(TH - 1) + kTileW <= PSZ && dz_row<1>(TH - 1) + kTileW <= PSZ && (PSZ / 2) % 2 == 1, "dz plane layout");

struct WgradParams {
  WgradArgs a;
  int Ho, Wo;
  int CC, nchunks, G;
  int rows, cols, RS, PS;  // x halo tile in LDS
  int shift;               // LDS column of the tile's first column (keeps the interior 8-byte aligned)
  int inv_rows;            // ceil(65536 / rows): exact division of small line numbers
  int tiles_x, tiles_y, items;
  int kgroups;
  long db_offset;
  long group_stride;       // floats between filter groups in the dw partial area
  int nxi, nxh;            // fast path: staging rounds the tile really needs (<= NXI, NXH)
  unsigned x_bytes, dy_bytes;   // fast path: tensor sizes (below 2 GiB) for the range-checked loads
};

__device__ __forceinline__ float act_deriv(int act, float out) {
  if (act == ACT_SIGMOID) return out * (1.0f - out);
  if (act == ACT_RELU) return out > 0.0f ? 1.0f : 0.0f;
  return 1.0f;
}

__device__ __forceinline__ float dz_value(const WgradArgs &a, int Ho, int Wo, int n, int k, int i, int j) {
  int o;
  if (a.pool == 2) {
    o = ((n * a.K + k) * (Ho >> 1) + (i >> 1)) * (Wo >> 1) + (j >> 1);
    const unsigned char f = a.idx[o];
    if ((f & kIdxPosMask) != (unsigned char)(((i & 1) << 1) | (j & 1))) return 0.0f;
    if (a.act == ACT_RELU_FLAGGED) return (f & kIdxInactive) ? 0.0f : a.dy[o];
  } else {
    o = ((n * a.K + k) * Ho + i) * Wo + j;
  }
  float g = a.dy[o];
  if (a.act != ACT_IDENTITY) g *= act_deriv(a.act, a.y[o]);
  return g;
}

__host__ __device__ __forceinline__ bool reads_output(int act) { return act == ACT_SIGMOID || act == ACT_RELU; }

// Registers that carry one tile from global memory to LDS (fast path).
template <int MTF, int POOL, int XI, int XH>
struct TileRegs {
  static constexpr int DZR = POOL == 2 ? MTF : 4 * MTF;   // staging rounds over the filter planes
  float4 xi[XI];
  float xh[XH];
  float4 dyv[DZR], yv[DZR];
  uchar4 iv[DZR];
};

// grid: x = G * nchunks, y = filter groups of MTF*16
// FAST: 0 = element-wise staging; 1 = vector staging with NXI / NXH rounds; 2 = vector staging
// of a halo tile small enough for ONE round of each (a few channels of a small filter): the
// loader registers and per-slot indices of the other rounds are gone, which buys two more
// resident workgroups per CU for a kernel whose rate follows its occupancy.
template <int MTF, int NTT, int POOL, int FAST>
__global__ __launch_bounds__(kThreads) void wgrad_kernel(const WgradParams p) {
  constexpr int XI = FAST == 2 ? 1 : NXI, XH = FAST == 2 ? 1 : NXH;
  extern __shared__ float lds[];
  const WgradArgs &a = p.a;
  float *xs = lds;                 // [CC][PS]
  float *dzs = xs + p.CC * p.PS;   // [filters of the group][PSZ]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, kq = lane >> 4;
  const int gidx = blockIdx.x % p.G, chunk = blockIdx.x / p.G;
  const int k0 = blockIdx.y * (MTF * 16);
  const int kcount = min(MTF * 16, a.K - k0);   // filters this group really has
  const int c0 = chunk * p.CC;
  const int RSf = a.R * a.S;
  const int lines = p.CC * p.rows;
  constexpr int RW = TH / 4;                    // rows per wave
  constexpr int DZR = TileRegs<MTF, POOL, XI, XH>::DZR;

  floatx4 acc[MTF][NTT];
#pragma unroll
  for (int mf = 0; mf < MTF; ++mf)
#pragma unroll
    for (int nt = 0; nt < NTT; ++nt) acc[mf][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
  float dbacc[FAST ? DZR : MTF * 16];
#pragma unroll
  for (int k = 0; k < (FAST ? DZR : MTF * 16); ++k) dbacc[k] = 0.0f;

  // B operand: lane's tap of N-tile nt -> offset inside the halo tile
  int tapoff[NTT];
#pragma unroll
  for (int nt = 0; nt < NTT; ++nt) {
    const int tap = nt * 16 + i16;
    const int cl = tap / RSf, rs = tap - cl * RSf;
    const int r = rs / a.S, s = rs - r * a.S;
    tapoff[nt] = (cl < p.CC) ? cl * p.PS + r * p.RS + s + p.shift : 0;
  }
  // A operand: lane's filter plane of M-tile mf (clipped: surplus rows are never stored)
  int fplane[MTF];
#pragma unroll
  for (int mf = 0; mf < MTF; ++mf) fplane[mf] = min(mf * 16 + i16, kcount - 1) * PSZ;

  TileRegs<MTF, POOL, XI, XH> tr;

  // ---- fast path: everything about a thread's staging slots that does not depend on the
  // tile (which element of the tile it moves, where it lands in LDS) is worked out once here;
  // per tile only a scalar base and a few range checks remain.
  constexpr int kUnused = -(1 << 20);
  const int j4 = 4 * (tid & 7);      // interior: first column of the thread's 16-byte group
  int xo[XI], xl[XI], xrow[XI];   // interior slots: global offset from the tile origin, LDS offset, tile row
  int ho[XH], hl[XH], hrow[XH], hcol[XH];
  int dzo[DZR], dzl[DZR];            // dz slots: global offset from the tile's first pooled element, LDS offset
  bool dzk[DZR];
  int du = 0, dv = 0;
  // The fast path reads through range-checked buffer loads: a slot that does not exist (beyond
  // the tile, the last channel or the filter group) keeps an offset past the end of the tensor
  // and reads zeros, as do rows and columns outside the image on the edge tiles.  Interior tiles
  // need no per-slot arithmetic at all: fixed per-thread offset + the tile's scalar offset.
  constexpr unsigned kOob = 0x80000000u;
  const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.x), 0, (int)p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_dy = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.dy), 0, (int)p.dy_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.y ? a.y : a.dy), 0, (int)p.dy_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_idx = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<unsigned char *>(a.idx ? a.idx : reinterpret_cast<const unsigned char *>(a.dy)), 0, (int)(p.dy_bytes >> 2), 0x00020000);
  if (FAST) {
#pragma unroll
    for (int it = 0; it < XI; ++it) {
      const int e = tid + it * kThreads;
      const int line = e >> 3;
      const int cl = (line * p.inv_rows) >> 16, row = line - cl * p.rows;
      const bool ok = line < lines && c0 + cl < a.C;
      xo[it] = ok ? 4 * ((cl * a.H + row) * a.W + j4 + a.pad) : (int)kOob;   // bytes from the halo tile's first element
      xl[it] = cl * p.PS + row * p.RS + a.pad + p.shift + j4;
      xrow[it] = ok ? row : kUnused;
      if (line >= lines) xl[it] = -1;   // slot beyond the tile: nothing to store
    }
    const int nh = a.S - 1;
#pragma unroll
    for (int it = 0; it < XH; ++it) {
      const int e = tid + it * kThreads;
      const int line = nh > 0 ? e / nh : lines, hc = nh > 0 ? e - line * nh : 0;
      const int cl = (line * p.inv_rows) >> 16, row = line - cl * p.rows;
      const bool ok = line < lines && c0 + cl < a.C;
      hcol[it] = hc < a.pad ? hc - a.pad : kTileW + hc - a.pad;   // column relative to the tile's first output column
      ho[it] = ok ? 4 * ((cl * a.H + row) * a.W + hcol[it] + a.pad) : (int)kOob;   // never negative: the range check reads it as unsigned
      hl[it] = line < lines ? cl * p.PS + row * p.RS + (hc < a.pad ? hc : kTileW + hc) + p.shift : -1;
      hrow[it] = ok ? row : kUnused;
    }
    if (POOL == 2) {
      const int q = tid & 15;
      du = q >> 2;
      dv = (q & 3) * 4;
#pragma unroll
      for (int rd = 0; rd < DZR; ++rd) {
        const int k = rd * 16 + (tid >> 4);
        dzk[rd] = k < kcount;
        dzo[rd] = dzk[rd] ? ((k0 + k) * (p.Ho >> 1) + du) * (p.Wo >> 1) + dv : (int)(kOob >> 2);   // element offset
        dzl[rd] = k * PSZ + dz_row<POOL>(2 * du) + 2 * dv;
      }
    } else {
      const int q = tid & 63;
      du = q >> 3;
      dv = (q & 7) * 4;
#pragma unroll
      for (int rd = 0; rd < DZR; ++rd) {
        const int k = rd * 4 + (tid >> 6);
        dzk[rd] = k < kcount;
        dzo[rd] = dzk[rd] ? ((k0 + k) * p.Ho + du) * p.Wo + dv : (int)(kOob >> 2);
        dzl[rd] = k * PSZ + dz_row<POOL>(du) + dv;
      }
    }
  }

  // ---- fast path, step 1: global -> registers for one tile
  auto ldx4 = [&](const __amdgpu_buffer_rsrc_t &r, int voff, unsigned soff) __attribute__((always_inline)) {
    const floatx4 v = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(r, voff, (int)soff, 0));
    return make_float4(v[0], v[1], v[2], v[3]);
  };
  auto load_tile = [&](int item) {
    const int tx = item % p.tiles_x;
    const int ty = (item / p.tiles_x) % p.tiles_y;
    const int n = item / (p.tiles_x * p.tiles_y);
    const int oy0 = ty * TH, ox0 = tx * kTileW;
    const int gy0 = oy0 - a.pad;                                            // image row of the halo tile's first row
    const unsigned xbase = 4u * ((unsigned)(n * a.C + c0) * a.H * a.W);     // bytes to (n, c0, 0, 0)
    const int torg = 4 * (gy0 * a.W + ox0 - a.pad);                         // bytes to the halo tile's first element inside a plane (negative on the top/left edge)
    // interior tile: every row and column of the halo tile lies inside the image
    const bool inner = gy0 >= 0 && gy0 + p.rows <= a.H && ox0 - a.pad >= 0 && ox0 - a.pad + p.cols <= a.W;
    if (inner) {
      const unsigned so = xbase + (unsigned)torg;
      // every round is issued: slots the tile does not have carry the out-of-range offset and cost
      // one load instruction that never reaches memory (cheaper than a branch with register copies)
#pragma unroll
      for (int it = 0; it < XI; ++it) tr.xi[it] = ldx4(rs_x, xo[it], so);
#pragma unroll
      for (int it = 0; it < XH; ++it)
        tr.xh[it] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_x, ho[it], (int)so, 0));
    } else {
      const bool col_ok = ox0 + j4 < a.W;
#pragma unroll
      for (int it = 0; it < XI; ++it) {
        const bool ok = (unsigned)(gy0 + xrow[it]) < (unsigned)a.H && col_ok;
        tr.xi[it] = ldx4(rs_x, ok ? xo[it] + torg : (int)kOob, xbase);
      }
#pragma unroll
      for (int it = 0; it < XH; ++it) {
        const bool ok = (unsigned)(gy0 + hrow[it]) < (unsigned)a.H && (unsigned)(ox0 + hcol[it]) < (unsigned)a.W;
        tr.xh[it] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_x, ok ? ho[it] + torg : (int)kOob, (int)xbase, 0));
      }
    }
    unsigned dbase;   // element offset of the tile's first (pooled) output element of filter 0
    bool in;
    if (POOL == 2) {
      const int Hp = p.Ho >> 1, Wp = p.Wo >> 1;
      dbase = ((unsigned)n * a.K * Hp + (oy0 >> 1)) * Wp + (ox0 >> 1);
      in = (oy0 >> 1) + du < Hp && (ox0 >> 1) + dv < Wp;
    } else {
      dbase = ((unsigned)n * a.K * p.Ho + oy0) * p.Wo + ox0;
      in = oy0 + du < p.Ho && ox0 + dv < p.Wo;
    }
#pragma unroll
    for (int rd = 0; rd < DZR; ++rd) {
      const int eo = in ? dzo[rd] : (int)(kOob >> 2);
      tr.dyv[rd] = ldx4(rs_dy, 4 * eo, 4u * dbase);
      if (reads_output(a.act)) tr.yv[rd] = ldx4(rs_y, 4 * eo, 4u * dbase);
      if (POOL == 2) tr.iv[rd] = __builtin_bit_cast(uchar4, __builtin_amdgcn_raw_buffer_load_b32(rs_idx, eo, (int)dbase, 0));
    }
  };

  // ---- fast path, step 2: registers -> LDS (dz is formed here)
  // `actc` carries the activation as a compile-time constant: with a run-time one the compiler
  // evaluates every derivative form for every element and selects afterwards
  auto store_tile_as = [&](auto actc) {
    constexpr int ACT = decltype(actc)::value;
#pragma unroll
    for (int it = 0; it < XI; ++it) {
      if (it < p.nxi && xl[it] >= 0) {
        float2 *d = reinterpret_cast<float2 *>(xs + xl[it]);
        d[0] = make_float2(tr.xi[it].x, tr.xi[it].y);
        d[1] = make_float2(tr.xi[it].z, tr.xi[it].w);
      }
    }
#pragma unroll
    for (int it = 0; it < XH; ++it)
      if (it < p.nxh && hl[it] >= 0) xs[hl[it]] = tr.xh[it];
#pragma unroll
    for (int rd = 0; rd < DZR; ++rd) {
      if (!dzk[rd]) continue;
      const float gv[4] = {tr.dyv[rd].x, tr.dyv[rd].y, tr.dyv[rd].z, tr.dyv[rd].w};
      const float ov[4] = {tr.yv[rd].x, tr.yv[rd].y, tr.yv[rd].z, tr.yv[rd].w};
      float g[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) g[e] = reads_output(ACT) ? gv[e] * act_deriv(ACT, ov[e]) : gv[e];
      float *d = dzs + dzl[rd];
      if (POOL == 2) {
        const unsigned char fl[4] = {tr.iv[rd].x, tr.iv[rd].y, tr.iv[rd].z, tr.iv[rd].w};
        unsigned char pos[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (ACT == ACT_RELU_FLAGGED && (fl[e] & kIdxInactive)) g[e] = 0.0f;
          pos[e] = fl[e] & kIdxPosMask;   // slots outside the image hold dy = 0
        }
        // the four 2x2 windows are cleared with plain stores, then each gradient is dropped at its
        // arg-max position (LDS writes of one wavefront land in program order): one address
        // computation per element instead of four compare/select pairs
#pragma unroll
        for (int wa = 0; wa < 2; ++wa)
#pragma unroll
          for (int e = 0; e < 4; ++e) *reinterpret_cast<float2 *>(d + wa * kTileW + 2 * e) = make_float2(0.0f, 0.0f);
#pragma unroll
        for (int e = 0; e < 4; ++e) d[2 * e + (pos[e] >> 1) * kTileW + (pos[e] & 1)] = g[e];
        dbacc[rd] += (g[0] + g[1]) + (g[2] + g[3]);
      } else {
        reinterpret_cast<float2 *>(d)[0] = make_float2(g[0], g[1]);
        reinterpret_cast<float2 *>(d)[1] = make_float2(g[2], g[3]);
        dbacc[rd] += (g[0] + g[1]) + (g[2] + g[3]);
      }
    }
  };
  auto store_tile = [&]() {
    if (a.act == ACT_SIGMOID) store_tile_as(std::integral_constant<int, ACT_SIGMOID>{});
    else if (a.act == ACT_RELU) store_tile_as(std::integral_constant<int, ACT_RELU>{});
    else if (a.act == ACT_RELU_FLAGGED) store_tile_as(std::integral_constant<int, ACT_RELU_FLAGGED>{});
    else store_tile_as(std::integral_constant<int, ACT_IDENTITY>{});
  };

  // ---- generic path: element-wise staging straight into LDS (any shape, any alignment)
  auto stage_generic = [&](int item) {
    const int tx = item % p.tiles_x;
    const int ty = (item / p.tiles_x) % p.tiles_y;
    const int n = item / (p.tiles_x * p.tiles_y);
    const int oy0 = ty * TH, ox0 = tx * kTileW;
#pragma unroll
    for (int k = 0; k < MTF * 16; ++k) {
      if (k < kcount) {
        const int col = tid & 31, row = tid >> 5;
        const int gi = oy0 + row, gj = ox0 + col;
        float v = 0.0f;
        if (gi < p.Ho && gj < p.Wo) v = dz_value(a, p.Ho, p.Wo, n, k0 + k, gi, gj);
        dzs[k * PSZ + dz_row<POOL>(row) + col] = v;
        if constexpr (!FAST) dbacc[k] += v;
      }
    }
    const int total = lines * p.cols;
    int col = tid % p.cols;
    int q = tid / p.cols;
    int row = q % p.rows, cl = q / p.rows;
    const int dcol = kThreads % p.cols, dq = kThreads / p.cols;
    for (int e = tid; e < total; e += kThreads) {
      const int gi = oy0 - a.pad + row, gj = ox0 - a.pad + col, ci = c0 + cl;
      float v = 0.0f;
      if (ci < a.C && gi >= 0 && gi < a.H && gj >= 0 && gj < a.W)
        v = a.x[((long)(n * a.C + ci) * a.H + gi) * a.W + gj];
      xs[cl * p.PS + row * p.RS + col + p.shift] = v;
      col += dcol;
      row += dq;
      if (col >= p.cols) { col -= p.cols; ++row; }
      while (row >= p.rows) { row -= p.rows; ++cl; }
    }
  };

  // Tile order is XCD-aware: workgroup ids are dealt round-robin to the 8 XCDs, each with its
  // own L2, so every XCD gets one contiguous eighth of the tiles and its workgroups stride
  // through it together: tiles in flight on an XCD are neighbours (shared halo rows and the
  // two halves of shared cache lines meet in that XCD's L2).
  const int nx = (p.G % 8 == 0) ? 8 : 1;
  const int xcd = gidx % nx, slot = gidx / nx, slots = p.G / nx;
  const int per_xcd = (p.items + nx - 1) / nx;
  const int item_base = xcd * per_xcd, item_lim = min(p.items, item_base + per_xcd);
  if (FAST && item_base + slot < item_lim) load_tile(item_base + slot);
  for (int item = item_base + slot; item < item_lim; item += slots) {
    __syncthreads();   // the previous tile's MFMA reads are done
    if (FAST) store_tile(); else stage_generic(item);
    __syncthreads();
    if (FAST && item + slots < item_lim) load_tile(item + slots);   // in flight during the MFMA loop
    // ---- MFMA: 4 neighbouring pixels per step.  Operand fragments are double-buffered in
    // registers: the LDS reads of step t+1 are issued before the MFMAs of step t.
    {
      float af[2][MTF], bf[2][NTT];
      static_assert(RW == 2, "dz_row(wave * RW + rr) = dz_row(wave * RW) + dz_row(rr) needs an even first row");
      const float *za = dzs + dz_row<POOL>(wave * RW) + kq;
      const float *xb = xs + (wave * RW) * p.RS + kq;
      auto load_frags = [&](auto bufc, int rr, int cg) {
        constexpr int B_ = decltype(bufc)::value;
#pragma unroll
        for (int mf = 0; mf < MTF; ++mf) af[B_][mf] = za[fplane[mf] + dz_row<POOL>(rr) + 4 * cg];
#pragma unroll
        for (int nt = 0; nt < NTT; ++nt) bf[B_][nt] = xb[tapoff[nt] + rr * p.RS + 4 * cg];
      };
      auto mfma_frags = [&](auto bufc) {
        constexpr int B_ = decltype(bufc)::value;
#pragma unroll
        for (int mf = 0; mf < MTF; ++mf)
#pragma unroll
          for (int nt = 0; nt < NTT; ++nt)
            acc[mf][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[B_][mf], bf[B_][nt], acc[mf][nt], 0, 0, 0);
      };
      using I0 = std::integral_constant<int, 0>;
      using I1 = std::integral_constant<int, 1>;
      load_frags(I0{}, 0, 0);
#pragma unroll
      for (int t = 0; t < RW * 8; t += 2) {
        load_frags(I1{}, (t + 1) >> 3, (t + 1) & 7);
        __builtin_amdgcn_sched_barrier(0);
        mfma_frags(I0{});
        __builtin_amdgcn_sched_barrier(0);
        if (t + 2 < RW * 8) load_frags(I0{}, (t + 2) >> 3, (t + 2) & 7);
        __builtin_amdgcn_sched_barrier(0);
        mfma_frags(I1{});
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }

  // ---- add the four wavefronts' accumulators in a fixed order: (w0 + w2) + (w1 + w3)
  constexpr int BLK = MTF * NTT * 256;   // floats per accumulator block
  float *red = lds;                      // 2 * BLK floats (the host plans LDS for it)
  __syncthreads();
  if (wave >= 2) {
#pragma unroll
    for (int mf = 0; mf < MTF; ++mf)
#pragma unroll
      for (int nt = 0; nt < NTT; ++nt)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[(wave - 2) * BLK + ((mf * NTT + nt) * 4 + v) * 64 + lane] = acc[mf][nt][v];
  }
  __syncthreads();
  if (wave < 2) {
#pragma unroll
    for (int mf = 0; mf < MTF; ++mf)
#pragma unroll
      for (int nt = 0; nt < NTT; ++nt)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[mf][nt][v] += red[wave * BLK + ((mf * NTT + nt) * 4 + v) * 64 + lane];
  }
  __syncthreads();
  if (wave == 1) {
#pragma unroll
    for (int mf = 0; mf < MTF; ++mf)
#pragma unroll
      for (int nt = 0; nt < NTT; ++nt)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[((mf * NTT + nt) * 4 + v) * 64 + lane] = acc[mf][nt][v];
  }
  __syncthreads();
  if (wave == 0) {
    // partial block of this workgroup: [chunk*G + g][mf][nt][v][lane], per filter group
    float *dst = a.partial + (long)blockIdx.y * p.group_stride + (long)(chunk * p.G + gidx) * BLK;
#pragma unroll
    for (int mf = 0; mf < MTF; ++mf)
#pragma unroll
      for (int nt = 0; nt < NTT; ++nt)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int o = ((mf * NTT + nt) * 4 + v) * 64 + lane;
          dst[o] = acc[mf][nt][v] + red[o];
        }
  }

  // ---- db partials: one value per workgroup and filter, [g][K]
  if (chunk == 0) {
    float *dbs = lds + 2 * BLK;   // [4][MTF*16]
    if (FAST) {
#pragma unroll
      for (int rd = 0; rd < DZR; ++rd) {
        float s = dbacc[rd];
        if (POOL == 2) {
#pragma unroll
          for (int off = 8; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);   // 16 lanes share a filter
          if ((lane & 15) == 0) dbs[rd * 16 + (tid >> 4)] = s;
        } else {
#pragma unroll
          for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);  // a wavefront shares a filter
          if (lane == 0) dbs[rd * 4 + wave] = s;
        }
      }
      __syncthreads();
      if (tid < kcount) a.partial[p.db_offset + (long)gidx * a.K + k0 + tid] = dbs[tid];
    } else {
#pragma unroll
      for (int k = 0; k < MTF * 16; ++k) {
        float s = dbacc[k];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
        if (lane == 0) dbs[wave * (MTF * 16) + k] = s;
      }
      __syncthreads();
      if (tid < kcount)
        a.partial[p.db_offset + (long)gidx * a.K + k0 + tid] =
            (dbs[tid] + dbs[2 * MTF * 16 + tid]) + (dbs[MTF * 16 + tid] + dbs[3 * MTF * 16 + tid]);
    }
  }
}

// Second pass over the partial blocks.  A block is laid out [mf][nt][v][lane] and a lane's 16
// neighbours are 16 consecutive taps of one filter, i.e. (inside a channel chunk) consecutive
// elements of dw.  A workgroup owns 16 such floats of the block layout: four threads read them
// as 16-byte groups, 64 slices of the partial list run in parallel, sums are kept in double
// and combined in a fixed order.  Blocks past the dw part sum the bias partials [g][K].
constexpr int kRedSlices = kThreads / 4;
__device__ __forceinline__ void wgrad_reduce_block(const WgradReduceArgs &a, const WgradPlan &plan, long group_stride,
                                                   int kgroups, int block) {
  __shared__ double red[kRedSlices][17];
  __shared__ double red2[4][17];
  const int tid = threadIdx.x, t4 = tid & 3, slice = tid >> 2;
  const int RSf = a.R * a.S;
  const int rows = plan.MTF * plan.NTT * 4;           // 64-float rows of a block
  const int per_chunk = rows * 4;                     // workgroups per (filter group, chunk)
  const int nblk_dw = kgroups * plan.nchunks * per_chunk;
  const long blockf = (long)rows * 64;
  int blk = block;
  double sum[4] = {0.0, 0.0, 0.0, 0.0};
  const bool is_dw = blk < nblk_dw;
  int grp = 0, chunk = 0, within0 = 0;
  if (is_dw) {
    grp = blk / (plan.nchunks * per_chunk);
    blk -= grp * plan.nchunks * per_chunk;
    chunk = blk / per_chunk;
    within0 = (blk - chunk * per_chunk) * 16;
    const long base = (long)grp * group_stride + (long)chunk * plan.n_partials * blockf + within0 + 4 * t4;
    // loads first, sums after: four independent 16-byte loads are in flight per thread
    for (int p0 = slice; p0 < plan.n_partials; p0 += 4 * kRedSlices) {
      float4 pv[4], nv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int pidx = p0 + u * kRedSlices;
        const bool in = pidx < plan.n_partials;
        const long o = base + (in ? pidx : 0) * blockf;
        pv[u] = *reinterpret_cast<const float4 *>(a.pos + o);
        nv[u] = a.neg ? *reinterpret_cast<const float4 *>(a.neg + o) : make_float4(0.f, 0.f, 0.f, 0.f);
        if (!in) { pv[u] = make_float4(0.f, 0.f, 0.f, 0.f); nv[u] = pv[u]; }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        sum[0] += (double)pv[u].x - (double)nv[u].x;
        sum[1] += (double)pv[u].y - (double)nv[u].y;
        sum[2] += (double)pv[u].z - (double)nv[u].z;
        sum[3] += (double)pv[u].w - (double)nv[u].w;
      }
    }
  } else {
    const int k = (blk - nblk_dw) * 16 + 4 * t4;
    // same scheme: the loads of four partial blocks are issued before anything is added
    for (int p0 = slice; p0 < plan.n_partials; p0 += 4 * kRedSlices) {
      float pv[4][4], nv[4][4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int pidx = p0 + u * kRedSlices;
        const bool in = pidx < plan.n_partials;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bool ok = in && k + j < a.K;
          const long o = plan.db_offset + (ok ? (long)pidx * a.K + k + j : 0);
          pv[u][j] = a.pos[o];
          nv[u][j] = a.neg ? a.neg[o] : 0.0f;
          if (!ok) { pv[u][j] = 0.0f; nv[u][j] = 0.0f; }
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int j = 0; j < 4; ++j) sum[j] += (double)pv[u][j] - (double)nv[u][j];
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) red[slice][4 * t4 + j] = sum[j];
  __syncthreads();
  if (tid < 64) {   // four threads per output, 16 slices each
    const int part = tid >> 4, o16 = tid & 15;
    double s = 0.0;
#pragma unroll
    for (int q = 0; q < kRedSlices / 4; ++q) s += red[part * (kRedSlices / 4) + q][o16];
    red2[part][o16] = s;
  }
  __syncthreads();
  if (tid < 16) {
    const double s = (red2[0][tid] + red2[1][tid]) + (red2[2][tid] + red2[3][tid]);
    const float gval = (float)(s * (double)a.scale);
    if (is_dw) {
      // position in the block layout -> (filter, channel, tap)
      const int within = within0 + tid;
      const int row = within >> 6, lane = within & 63;
      const int v = row & 3, nt = (row >> 2) % plan.NTT, mf = (row >> 2) / plan.NTT;
      const int m = mf * 16 + (lane >> 4) * 4 + v, tap = nt * 16 + (lane & 15);
      const int cl = tap / RSf, rs = tap - cl * RSf;
      const int ko = grp * plan.MTF * 16 + m, ci = chunk * plan.CC + cl;
      if (cl < plan.CC && ci < a.C && ko < a.K) {
        const long o = ((long)ko * a.C + ci) * RSf + rs;
        if (a.dw) a.dw[o] = gval;
        if (a.w_update) update_param(a.w_update + o, a.w_vel ? a.w_vel + o : nullptr, gval, a.step, a.mu, a.w_decay);
      }
    } else {
      const int k = (blk - nblk_dw) * 16 + tid;
      if (k < a.K) {
        if (a.db) a.db[k] = gval;
        if (a.b_update) update_param(a.b_update + k, a.b_vel ? a.b_vel + k : nullptr, gval, a.step, a.mu, 0.0f);
      }
    }
  }
}

__global__ __launch_bounds__(kThreads) void wgrad_reduce_kernel(const WgradReduceArgs a, const WgradPlan plan,
                                                               long group_stride, int kgroups) {
  wgrad_reduce_block(a, plan, group_stride, kgroups, blockIdx.x);
}

inline long reduce_group_stride(const WgradPlan &plan) {
  return (long)plan.nchunks * plan.n_partials * ((long)plan.MTF * plan.NTT * 256);
}
inline int reduce_kgroups(const WgradReduceArgs &a, const WgradPlan &plan) { return (a.K + plan.MTF * 16 - 1) / (plan.MTF * 16); }
inline int reduce_blocks(const WgradReduceArgs &a, const WgradPlan &plan) {
  return reduce_kgroups(a, plan) * plan.nchunks * plan.MTF * plan.NTT * 16 + (a.K + 15) / 16;
}

// The step's closing kernel: workgroup ranges [start[j], start[j+1]) belong to job j; jobs are the
// filter-gradient reductions, then the column sums, then the mean loss.
struct StepTailParams {
  StepTail t;
  int start[StepTail::kMaxReduce + StepTail::kMaxColsum + 2];
  long group_stride[StepTail::kMaxReduce];
  int kgroups[StepTail::kMaxReduce];
};
__global__ __launch_bounds__(kThreads) void step_tail_kernel(const StepTailParams p) {
  const int b = blockIdx.x;
  int j = 0;
  while (b >= p.start[j + 1]) ++j;   // uniform; at most a dozen jobs
  const int blk = b - p.start[j];
  if (j < p.t.n_reduce) {
    wgrad_reduce_block(p.t.reduce[j].a, p.t.reduce[j].plan, p.group_stride[j], p.kgroups[j], blk);
  } else if (j < p.t.n_reduce + p.t.n_colsum) {
    const StepTail::Colsum &c = p.t.colsum[j - p.t.n_reduce];
    colsum_block(c.A, c.M, c.N, c.out, c.update, c.step, c.vel, c.mu, blk);
  } else {
    mean_block(p.t.rowloss, p.t.rows, p.t.loss);
  }
}

inline int round_up_mod(int v, int m, int r) {
  int x = v - (v % m) + r;
  if (x < v) x += m;
  return x;
}

const int kNttChoices[] = {2, 5, 7, 9};

inline int pick_ntt(int tiles) {
  for (int c : kNttChoices)
    if (tiles <= c) return c;
  return 0;
}

struct Geom {
  int rows, cols, RS, PS, shift;
};

inline Geom x_geom(int R, int S, int pad) {
  Geom g;
  g.rows = TH + R - 1;
  g.cols = kTileW + S - 1;
  g.shift = pad & 1;
  // A 16-tap operand tile touches consecutive (channel, filter row) lines of the halo tile,
  // S + 1 neighbouring columns of each (tap s plus the two pixels of a half wave): spacing the
  // lines S + 1 (rounded up to even) banks apart keeps those reads free of bank conflicts.
  const int sp = (S + 2) & ~1;
  g.RS = round_up_mod(g.cols + g.shift, 32, sp % 32);
  g.PS = round_up_mod(g.RS * g.rows, 32, (sp * R) % 32);
  if (g.PS & 1) ++g.PS;   // keeps 8-byte alignment of the vector stores
  return g;
}

}  // namespace

bool plan_wgrad(int N, int C, int H, int W, int K, int R, int S, int pad, int pool, WgradPlan *plan, bool shared_launch) {
  const int Ho = H + 2 * pad - R + 1, Wo = W + 2 * pad - S + 1;
  const int RSf = R * S;
  // channels per chunk: minimise (chunks x tap tiles) with at most 9 tap tiles
  int best_cc = 0, best_cost = 0, best_ntt = 0;
  for (int cc = 1; cc <= (C < 16 ? C : 16); ++cc) {
    const int ntt = pick_ntt((cc * RSf + 15) / 16);
    if (!ntt) break;
    const int cost = ((C + cc - 1) / cc) * ntt;
    if (!best_cc || cost <= best_cost) { best_cc = cc; best_cost = cost; best_ntt = ntt; }
  }
  if (!best_cc) return false;
  plan->CC = best_cc;
  plan->NTT = best_ntt;
  plan->nchunks = (C + best_cc - 1) / best_cc;
  plan->TH = TH;
  const Geom g = x_geom(R, S, pad);
  int mtf = (K + 15) / 16;
  if (mtf > 3) mtf = 3;
  for (;; --mtf) {
    const int planes = K < mtf * 16 ? K : mtf * 16;
    const size_t stage = (size_t)best_cc * g.PS + (size_t)planes * PSZ;
    const size_t reduce = (size_t)2 * mtf * best_ntt * 256 + 4 * mtf * 16;
    plan->lds_bytes = sizeof(float) * (stage > reduce ? stage : reduce);
    if (plan->lds_bytes <= 64 * 1024) break;
    if (mtf == 1) return false;
  }
  plan->MTF = mtf;
  const int tiles_x = (Wo + kTileW - 1) / kTileW, tiles_y = (Ho + TH - 1) / TH;
  const long items = (long)N * tiles_x * tiles_y;
  const int kgroups = (K + mtf * 16 - 1) / (mtf * 16);
  // persistent workgroups: as many as stay resident (LDS and register budget), at least two
  // tiles each where the problem is large enough
  long resident = (long)(chip().lds_bytes / plan->lds_bytes);
  // waves per SIMD that the kernel instance's registers (vector + accumulator, from the compiler's
  // resource report) leave room for; a grid beyond it would queue workgroups behind resident ones
  static const int kByRegs[2][3][4] = {
      // NTT =  2  5  7  9     (pooled staging)
      {{5, 4, 3, 3}, {4, 3, 2, 2}, {3, 2, 2, 2}},
      //                      (unpooled staging: more loader registers)
      {{4, 3, 3, 2}, {3, 2, 2, 2}, {2, 1, 1, 1}}};
  const int ntt_slot = best_ntt <= 2 ? 0 : (best_ntt <= 5 ? 1 : (best_ntt <= 7 ? 2 : 3));
  long by_regs = kByRegs[pool == 2 ? 0 : 1][mtf - 1][ntt_slot];
  // the one-round instances (two tap tiles, halo tile of at most 32 lines) carry far fewer loader registers
  static const int kByRegsOneRound[2][3] = {{7, 5, 4}, {5, 3, 2}};
  const int lines = best_cc * g.rows;
  if (best_ntt == 2 && lines * 8 <= kThreads && lines * (S - 1) <= kThreads) by_regs = kByRegsOneRound[pool == 2 ? 0 : 1][mtf - 1];
  if (resident > by_regs) resident = by_regs;
  if (resident < 1) resident = 1;
  const long cus = chip().cus;
  long G = cus * resident / ((long)plan->nchunks * kgroups);
  if (G < 1) G = 1;
  // fewer tiles than CUs: one tile per workgroup (what counts there is the length of the longest
  // workgroup, not the number of partial blocks)
  const long cap = items <= cus ? items : (items + 1) / 2;
  if (G > cap) G = cap;
  // layers the minimal-filtering kernel can take: its registers leave two workgroups per compute unit,
  // and every one of them should be resident from the start (the direct kernel copes with any G)
  if (wgrad_wino_shape(C, H, W, K, R, S, pad, pool) && mtf * 16 == K && best_cc == 16) {
    const long want = ((C == 32 && K == 32) || shared_launch) ? cus : 2 * cus;   // 32 x 32 filters: 36 KB per partial block; halving their number took 2 us off the step
    G = want < items ? want : items;
  }
  // the first-layer kernel keeps four workgroups per compute unit resident
  if (wgrad_fewch_shape(C, H, W, K, R, S, pad, pool) && mtf == 1 && best_ntt == 2 && best_cc == C) G = 4 * cus < items ? 4 * cus : items;
  if (G < 1) G = 1;
  plan->G = (int)G;
  plan->n_partials = plan->G;
  const size_t blockf = (size_t)mtf * plan->NTT * 256;
  const size_t group_stride = (size_t)plan->nchunks * plan->n_partials * blockf;
  plan->db_offset = group_stride * kgroups;
  plan->partial_floats = plan->db_offset + (size_t)plan->n_partials * K;
  return true;
}

namespace {

template <int MTF, int NTT>
hipError_t launch_wgrad_t(const WgradParams &p, const WgradPlan &plan, bool fast, hipStream_t stream) {
  dim3 grid((unsigned)(plan.G * plan.nchunks), (unsigned)p.kgroups, 1);
  if constexpr (NTT == 2) {
    if (fast && p.nxi <= 1 && p.nxh <= 1) {   // one staging round: the instance with the small loader
      if (p.a.pool == 2) hipLaunchKernelGGL((wgrad_kernel<MTF, NTT, 2, 2>), grid, dim3(kThreads), plan.lds_bytes, stream, p);
      else hipLaunchKernelGGL((wgrad_kernel<MTF, NTT, 1, 2>), grid, dim3(kThreads), plan.lds_bytes, stream, p);
      return hipGetLastError();
    }
  }
  if (fast && p.a.pool == 2)
    hipLaunchKernelGGL((wgrad_kernel<MTF, NTT, 2, 1>), grid, dim3(kThreads), plan.lds_bytes, stream, p);
  else if (fast)
    hipLaunchKernelGGL((wgrad_kernel<MTF, NTT, 1, 1>), grid, dim3(kThreads), plan.lds_bytes, stream, p);
  else
    hipLaunchKernelGGL((wgrad_kernel<MTF, NTT, 1, 0>), grid, dim3(kThreads), plan.lds_bytes, stream, p);
  return hipGetLastError();
}
template <int MTF>
hipError_t launch_wgrad_m(const WgradParams &p, const WgradPlan &plan, bool fast, hipStream_t stream) {
  switch (plan.NTT) {
  case 2: return launch_wgrad_t<MTF, 2>(p, plan, fast, stream);
  case 5: return launch_wgrad_t<MTF, 5>(p, plan, fast, stream);
  case 7: return launch_wgrad_t<MTF, 7>(p, plan, fast, stream);
  case 9: return launch_wgrad_t<MTF, 9>(p, plan, fast, stream);
  default: return hipErrorInvalidValue;
  }
}

inline bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

}  // namespace

hipError_t launch_wgrad(const WgradArgs &a, const WgradPlan &plan, hipStream_t stream) {
  if (wgrad_wino_applies(a, plan)) return launch_wgrad_wino(a, plan, stream);
  if (wgrad_fewch_applies(a, plan)) return launch_wgrad_fewch(a, plan, stream);
  WgradParams p;
  p.a = a;
  p.Ho = a.H + 2 * a.pad - a.R + 1;
  p.Wo = a.W + 2 * a.pad - a.S + 1;
  p.CC = plan.CC;
  p.nchunks = plan.nchunks;
  p.G = plan.G;
  const Geom g = x_geom(a.R, a.S, a.pad);
  p.rows = g.rows; p.cols = g.cols; p.RS = g.RS; p.PS = g.PS; p.shift = g.shift;
  p.inv_rows = (65536 + g.rows - 1) / g.rows;
  p.tiles_x = (p.Wo + kTileW - 1) / kTileW;
  p.tiles_y = (p.Ho + TH - 1) / TH;
  p.items = a.N * p.tiles_x * p.tiles_y;
  p.kgroups = (a.K + plan.MTF * 16 - 1) / (plan.MTF * 16);
  p.db_offset = (long)plan.db_offset;
  p.group_stride = (long)plan.nchunks * plan.n_partials * ((long)plan.MTF * plan.NTT * 256);
  // Vector staging needs whole 16-byte groups: image rows and output rows that are multiples
  // of 4 (8 pre-pool columns when pooling), aligned tensors, and a tile that fits the
  // prefetch registers.
  const int lines = plan.CC * g.rows;
  bool fast = (a.W % 4 == 0) && aligned16(a.x) && aligned16(a.dy) && (!reads_output(a.act) || aligned16(a.y)) &&
              lines * 8 <= NXI * kThreads && lines * (a.S - 1) <= NXH * kThreads;
  if (a.pool == 2) fast = fast && (p.Wo % 8 == 0) && ((reinterpret_cast<uintptr_t>(a.idx) & 3u) == 0);
  else fast = fast && (p.Wo % 4 == 0);
  // 32-bit byte offsets with an out-of-range marker at 2 GiB
  const long x_bytes = 4L * a.N * a.C * a.H * a.W, dy_bytes = 4L * a.N * a.K * (p.Ho / a.pool) * (p.Wo / a.pool);
  const long limit = (1L << 31) - (1L << 24);
  fast = fast && x_bytes < limit && dy_bytes < limit;
  p.x_bytes = (unsigned)(x_bytes < limit ? x_bytes : 0);
  p.dy_bytes = (unsigned)(dy_bytes < limit ? dy_bytes : 0);
  p.nxi = (lines * 8 + kThreads - 1) / kThreads;
  p.nxh = (lines * (a.S - 1) + kThreads - 1) / kThreads;
  switch (plan.MTF) {
  case 1: return launch_wgrad_m<1>(p, plan, fast, stream);
  case 2: return launch_wgrad_m<2>(p, plan, fast, stream);
  case 3: return launch_wgrad_m<3>(p, plan, fast, stream);
  default: return hipErrorInvalidValue;
  }
}

hipError_t launch_wgrad_reduce(const WgradReduceArgs &a, const WgradPlan &plan, hipStream_t stream) {
  if ((reinterpret_cast<uintptr_t>(a.pos) & 15u) || (a.neg && (reinterpret_cast<uintptr_t>(a.neg) & 15u))) return hipErrorInvalidValue;
  hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(reduce_blocks(a, plan)), dim3(kThreads), 0, stream, a, plan,
                     reduce_group_stride(plan), reduce_kgroups(a, plan));
  return hipGetLastError();
}

hipError_t launch_step_tail(const StepTail &t, hipStream_t stream) {
  if (t.n_reduce < 0 || t.n_reduce > StepTail::kMaxReduce || t.n_colsum < 0 || t.n_colsum > StepTail::kMaxColsum) return hipErrorInvalidValue;
  StepTailParams p;
  p.t = t;
  int jobs = 0, blocks = 0;
  for (int j = 0; j < t.n_reduce; ++j) {
    const WgradReduceArgs &a = t.reduce[j].a;
    if ((reinterpret_cast<uintptr_t>(a.pos) & 15u) || (a.neg && (reinterpret_cast<uintptr_t>(a.neg) & 15u))) return hipErrorInvalidValue;
    p.group_stride[j] = reduce_group_stride(t.reduce[j].plan);
    p.kgroups[j] = reduce_kgroups(a, t.reduce[j].plan);
    p.start[jobs++] = blocks;
    blocks += reduce_blocks(a, t.reduce[j].plan);
  }
  for (int j = 0; j < t.n_colsum; ++j) {
    p.start[jobs++] = blocks;
    blocks += (t.colsum[j].N + kColsumCols - 1) / kColsumCols;
  }
  if (t.loss) {
    p.start[jobs++] = blocks;
    blocks += 1;
  }
  if (blocks == 0) return hipSuccess;
  for (int j = jobs; j < StepTail::kMaxReduce + StepTail::kMaxColsum + 2; ++j) p.start[j] = blocks;
  hipLaunchKernelGGL(step_tail_kernel, dim3(blocks), dim3(kThreads), 0, stream, p);
  return hipGetLastError();
}

}  // namespace dllk
