// Forward 3x3 convolution of a layer with 16 or 32 channels in and out, ReLU and 2x2 max pooling
// (and the backward-data pass of such a layer) in the
// minimal-filtering form F(2x2, 3x3): every 2x2 block of outputs comes from a 4x4 input patch,
//   Y = At [ (G g Gt) .* (Bt d B) ] A,
// so that the 36 multiplications per output pixel, input channel and filter of the direct sum
// become 16 per 2x2 block = 4 per pixel.  The products over the input channels are the matrix
// part: for each of the 16 transform points p, M_p[tile][k] = sum_c V_p[tile][c] U_p[c][k] runs on
// fp32 MFMA (16 tiles x 16 filters x 4 channels per instruction); the transforms are additions
// on the vector pipe.  A 2x2 output block is exactly one pooling window, so bias, ReLU, the
// maximum and its position follow in registers and only the pooled map is stored.
//
// Tile: 8 x 32 outputs = 4 x 16 blocks per workgroup; wavefront w owns block row w; lane
// (i16, kq) transforms the patch of block column i16 for the channels kq, 4+kq, 8+kq, 12+kq (its
// MFMA A fragments) and ends up with the 16 point sums of blocks 4kq..4kq+3 for filter i16.
// Results differ from the direct sum by rounding only (a few 1e-7 of the output scale).
#include "dll_internal.h"

namespace dllk {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kWT = 256;
constexpr int kC = 16, kK = 16;          // channels in, filters
constexpr int kRS = 36;                  // row stride of the halo tile in LDS (34 columns used)
// GRP block rows per wavefront: 1 -> tiles of 8 x 32 outputs (10 halo rows), the only form in use (tiles of
// 16 x 32 with 18 halo rows, GRP 2, leave room for two workgroups per CU instead of three and measured slower).  Plane stride = 16 mod 32: the four channel groups of a wavefront land 16 banks apart.
template <int GRP> struct WinoGeom {
  static constexpr int kRows = 8 * GRP + 2;
  static constexpr int kPS = GRP == 2 ? kRows * kRS + 8 : kRows * kRS + 16;   // 656, 376
};

struct WinoParams {
  ConvEngineArgs a;
  int tiles_x, tiles_y, items, xcd;
};

// BWD: the backward-data pass of such a layer instead (the same sum with the filters rotated and
// transposed): the source is dz = unpool(dy) with the ReLU flags of the pooling bytes, formed while
// staging from the pooled gradient; the 2x2 output blocks are stored as they are.
// CCH: source channels in chunks of 16 (1 or 2): a chunk is staged, its filters transformed, its
// products added to the same accumulators; LDS holds one chunk at a time.
// KCH: filters in groups of 16 (1 or 2): with 2, every transformed patch is multiplied
// with both groups' filters (two accumulator sets, two resident workgroups per CU instead of three).
template <int GRP, bool BWD, int CCH, int KCH>
__global__ __launch_bounds__(kWT, (GRP == 2 || KCH == 2) ? 2 : 3) void conv3x3_wino_kernel(const WinoParams p) {
  constexpr int kKout = kK * KCH;
  static_assert(GRP == 1, "one block row per wavefront: the accumulators live across the channel chunks");
  constexpr int kCin = kC * CCH;
  constexpr int kRows = WinoGeom<GRP>::kRows, kPS = WinoGeom<GRP>::kPS, kTH = 8 * GRP;
  __shared__ __attribute__((aligned(16))) float xs[kC * kPS];       // [c][row][col], zero-padded halo tile
  __shared__ __attribute__((aligned(16))) float us[16 * kC * kKout];   // [point][c][k], transformed filters
  const ConvEngineArgs &a = p.a;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, kq = lane >> 4;

  // ---- filters of a channel chunk: U = G g Gt, one (channel, filter) pair per thread
  auto load_filters = [&](int c0) __attribute__((always_inline)) {
    const int c = tid >> 4;
#pragma unroll
    for (int kg = 0; kg < KCH; ++kg) {
    const int k = kg * kK + (tid & 15);
    // forward: w[k][c][r][s]; backward-data: source channel c is the layer's filter index and the
    // taps are rotated, g[r][s] = w[c][k][2 - r][2 - s]
    const float *g = BWD ? a.w + ((long)(c0 + c) * kKout + k) * 9 : a.w + ((long)k * kCin + c0 + c) * 9;
    float gv[9];
#pragma unroll
    for (int e = 0; e < 9; ++e) gv[e] = g[BWD ? 8 - e : e];
    float t[4][3];   // G g
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      t[0][j] = gv[j];
      t[1][j] = 0.5f * (gv[j] + gv[3 + j] + gv[6 + j]);
      t[2][j] = 0.5f * (gv[j] - gv[3 + j] + gv[6 + j]);
      t[3][j] = gv[6 + j];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float u0 = t[i][0], u1 = 0.5f * (t[i][0] + t[i][1] + t[i][2]), u2 = 0.5f * (t[i][0] - t[i][1] + t[i][2]), u3 = t[i][2];
      us[((4 * i + 0) * kC + c) * kKout + k] = u0;
      us[((4 * i + 1) * kC + c) * kKout + k] = u1;
      us[((4 * i + 2) * kC + c) * kKout + k] = u2;
      us[((4 * i + 3) * kC + c) * kKout + k] = u3;
    }
    }   // filter groups
  };
  if (CCH == 1) load_filters(0);
  float bias[KCH];
#pragma unroll
  for (int kg = 0; kg < KCH; ++kg) bias[kg] = a.bias ? a.bias[kg * kK + i16] : 0.0f;
  const int Hp = a.Hout >> 1, Wp = a.Wout >> 1;

  // Staging slots: 16 channels x 18 rows x 9 groups of four columns (36 >= 34; the last two are never
  // read), eleven rounds of 256 threads.  What does not depend on the tile is worked out once: the
  // byte offset from the halo tile's first element, the LDS offset, the row and the column group.
  // The loads are range-checked buffer loads of 16 bytes at 4-byte alignment: an offset past the end
  // of the tensor (or "negative", i.e. huge) reads zeros, which is what padding needs.
  constexpr int kSlots = kC * kRows * 9, kRounds = (kSlots + kWT - 1) / kWT;
  constexpr unsigned kOob = 0x80000000u;
  const __amdgpu_buffer_rsrc_t rs_x =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.src), 0, (int)(4u * (unsigned)a.N * kCin * a.Hin * a.Win), 0x00020000);
  int goff[kRounds], loff[kRounds], srow[kRounds], sq[kRounds];
#pragma unroll
  for (int it = 0; it < kRounds; ++it) {
    const int e = tid + it * kWT;
    const int c = e / (kRows * 9), rem = e - c * (kRows * 9);
    const int r = rem / 9, q = rem - r * 9;
    const bool in = e < kSlots;
    goff[it] = in ? 4 * ((c * a.Hin + r) * a.Win + 4 * q) : (int)kOob;
    loff[it] = in ? c * kPS + r * kRS + 4 * q : -1;
    srow[it] = r;
    sq[it] = q;
  }
  // Backward-data staging slots over the tile's pooled window (rows oy0/2 - 1 .. oy0/2 + kTH/2, columns
  // ox0/2 - 1 .. ox0/2 + 16): per (channel, pooled row) four groups of four aligned columns, read as
  // 16 bytes of gradient + 4 pooling bytes, and the two edge columns, read one by one.  Per slot: the
  // source offset from the window's first element, the LDS offset of entry (0, 0) of its (first)
  // window, which may lie outside the tile: bit a of `rows` says whether window row a is inside.
  constexpr int kPR = kTH / 2 + 2;
  constexpr int kVecSlots = kC * kPR * 4, kVecRounds = BWD ? (kVecSlots + kWT - 1) / kWT : 1;
  constexpr int kEdgeSlots = kC * kPR * 2;
  static_assert(kEdgeSlots <= kWT, "one round of edge slots");
  int voffs[kVecRounds], vwin[kVecRounds], vinfo[kVecRounds];   // vinfo: rows mask (bits 0-1), pr (bits 4-7), exists (bit 8)
  int eoffs = 0, ewin = 0, einfo = 0;                            // einfo: rows mask, pr, exists, bit 9: right edge
  if constexpr (BWD) {
    const int Hs = a.Hin >> 1, Ws = a.Win >> 1;
    auto rows_of = [&](int pr) { return (2 * pr - 1 >= 0 ? 1 : 0) | (2 * pr < kRows ? 2 : 0); };
#pragma unroll
    for (int it = 0; it < kVecRounds; ++it) {
      const int e = tid + it * kWT;
      const int c = e / (kPR * 4), rem = e - c * (kPR * 4);
      const int pr = rem >> 2, g = rem & 3;
      voffs[it] = (c * Hs + pr) * Ws + 1 + 4 * g;
      vwin[it] = c * kPS + (2 * pr - 1) * kRS + 2 * (1 + 4 * g) - 1;
      vinfo[it] = rows_of(pr) | (pr << 4) | (e < kVecSlots ? 1 << 8 : 0);
    }
    {
      const int e = tid;
      const int c = e / (kPR * 2), rem = e - c * (kPR * 2);
      const int pr = rem >> 1, right = rem & 1, pc = right ? 17 : 0;
      eoffs = (c * Hs + pr) * Ws + pc;
      ewin = c * kPS + (2 * pr - 1) * kRS + 2 * pc - 1;
      einfo = rows_of(pr) | (pr << 4) | (e < kEdgeSlots ? 1 << 8 : 0) | (right << 9);
    }
  }
  // global -> registers for one tile, registers -> LDS with the edge fixes.  (Issuing the loads one
  // tile ahead, across the transforms and products of the previous tile, measured slower: 92 vs 86 us
  // on the 128 x 128 layer; the two resident workgroups of a CU overlap each other's staging instead.)
  floatx4 v[kRounds];
  auto load_tile = [&](int item, int c0) __attribute__((always_inline)) {
    const int tx = item % p.tiles_x, ty = (item / p.tiles_x) % p.tiles_y, n = item / (p.tiles_x * p.tiles_y);
    const int oy0 = ty * kTH, ox0 = tx * 32;
    const int base = 4 * (((n * kCin + c0) * a.Hin + oy0 - 1) * a.Win + ox0 - 1);   // bytes; negative at the very first tile
    const bool left = ox0 == 0, right = ox0 + 32 >= a.Win;
    const bool inner_rows = oy0 >= 1 && oy0 + kTH + 1 <= a.Hin;
#pragma unroll
    for (int it = 0; it < kRounds; ++it) {
      int off = goff[it] + base;
      if (!inner_rows) {
        const int gi = oy0 - 1 + srow[it];
        if (gi < 0 || gi >= a.Hin) off = (int)kOob;
      }
      // the groups that overhang the image on the left / right are read one / three columns further
      // in, so that no access starts before the tensor or runs past its end
      if (left && sq[it] == 0) off += 4;
      if (right && sq[it] == 8) off -= 12;
      if (goff[it] == (int)kOob) off = (int)kOob;
      v[it] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rs_x, off, 0, 0));
    }
  };
  auto store_tile = [&](int item) __attribute__((always_inline)) {
    const int tx = item % p.tiles_x;
    const int ox0 = tx * 32;
    const bool left = ox0 == 0, right = ox0 + 32 >= a.Win;
#pragma unroll
    for (int it = 0; it < kRounds; ++it) {
      if (loff[it] < 0) continue;
      floatx4 t = v[it];
      if (left && sq[it] == 0) t = floatx4{0.0f, t[0], t[1], t[2]};    // column -1 of the image is padding
      if (right && sq[it] == 8) t = floatx4{t[3], 0.0f, 0.0f, 0.0f};   // column Win is padding (the two after it are never read)
      *reinterpret_cast<floatx4 *>(xs + loff[it]) = t;
    }
  };
  const int vb = p.xcd ? (int)(blockIdx.x & 7) * (int)(gridDim.x >> 3) + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
  for (int item0 = 0; item0 < p.items; item0 += gridDim.x) {
    // whole rounds: neighbouring tiles on one XCD (one L2); the last, partial round in launch order,
    // which spreads it evenly over the XCDs
    const int item = item0 + (item0 + (int)gridDim.x <= p.items ? vb : (int)blockIdx.x);
    if (item >= p.items) break;
    const int tx = item % p.tiles_x, ty = (item / p.tiles_x) % p.tiles_y, n = item / (p.tiles_x * p.tiles_y);
    const int oy0 = ty * kTH, ox0 = tx * 32;
    const int tr = wave;   // block row inside the tile
    floatx4 acc[KCH][16];
    const floatx4 zero = floatx4{0.f, 0.f, 0.f, 0.f};   // the first channel quartet starts the sums from it
#pragma unroll 1
    for (int chunk = 0; chunk < CCH; ++chunk) {
    const int c0 = chunk * kC;
    __syncthreads();   // the previous chunk's / tile's readers are done (first tile: the filters are in place)
    if constexpr (!BWD) {
      // the tile's loads go out ahead of the chunk's filter loads: one memory round trip for both
      load_tile(item, c0);
      if (CCH > 1) load_filters(c0);
      store_tile(item);
    } else {
      if (CCH > 1) load_filters(c0);
      // dz halo tile from the pooled gradient.  The tile is cleared with 16-byte stores; then every
      // pooled element drops its gradient at the recorded position of its window, if that entry lies
      // inside the tile and the unit is not flagged inactive.  All loads first, stores after.
      const int Hs = a.Hin >> 1, Ws = a.Win >> 1;   // pooled source size
      const long pbase = (((long)n * kCin + c0) * Hs + (oy0 >> 1) - 1) * Ws + (ox0 >> 1) - 1;
      float4 gv[kVecRounds];
      uchar4 fv[kVecRounds];
      bool vok[kVecRounds];
#pragma unroll
      for (int it = 0; it < kVecRounds; ++it) {
        const int pi = (oy0 >> 1) - 1 + ((vinfo[it] >> 4) & 15);
        vok[it] = ((vinfo[it] >> 8) & 1) && pi >= 0 && pi < Hs;
        const long o = vok[it] ? pbase + voffs[it] : 0;   // element 0 stands in (16-byte aligned like every group)
        gv[it] = *reinterpret_cast<const float4 *>(a.src + o);
        fv[it] = *reinterpret_cast<const uchar4 *>(a.src_idx + o);
      }
      bool eok;
      float ge;
      unsigned char fe;
      {
        const int pi = (oy0 >> 1) - 1 + ((einfo >> 4) & 15);
        const int pj = (ox0 >> 1) - 1 + (((einfo >> 9) & 1) ? 17 : 0);
        eok = ((einfo >> 8) & 1) && pi >= 0 && pi < Hs && pj >= 0 && pj < Ws;
        const long o = eok ? pbase + eoffs : 0;
        ge = a.src[o];
        fe = a.src_idx[o];
      }
      for (int e = tid; e < kC * kPS / 4; e += kWT) reinterpret_cast<floatx4 *>(xs)[e] = floatx4{0.f, 0.f, 0.f, 0.f};
      __syncthreads();
#pragma unroll
      for (int it = 0; it < kVecRounds; ++it) {
        if (!vok[it]) continue;
        const float g4[4] = {gv[it].x, gv[it].y, gv[it].z, gv[it].w};
        const unsigned char f4[4] = {fv[it].x, fv[it].y, fv[it].z, fv[it].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int pos = f4[j] & kIdxPosMask;
          if (!(f4[j] & kIdxInactive) && ((vinfo[it] >> (pos >> 1)) & 1)) xs[vwin[it] + 2 * j + (pos >> 1) * kRS + (pos & 1)] = g4[j];
        }
      }
      if (eok && !(fe & kIdxInactive)) {
        const int pos = fe & kIdxPosMask;
        // left edge: only window column 1 is inside the tile; right edge: only column 0
        const bool col_in = ((einfo >> 9) & 1) ? (pos & 1) == 0 : (pos & 1) == 1;
        if (col_in && ((einfo >> (pos >> 1)) & 1)) xs[ewin + (pos >> 1) * kRS + (pos & 1)] = ge;
      }
    }
    __syncthreads();
    {
      // Per channel quartet s: patch and filter fragments come from LDS in one batch, issued while the
      // previous quartet's 16 products run (two register sets), so that no product waits for its own read.
      float dA[4][4], dB[4][4], uA[KCH][16], uB[KCH][16];
      auto read_s = [&](int s, float (&d)[4][4], float (&u)[KCH][16]) __attribute__((always_inline)) {
        const float *d0 = xs + (4 * s + kq) * kPS + (2 * tr) * kRS + 2 * i16;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float2 lo = *reinterpret_cast<const float2 *>(d0 + i * kRS);
          const float2 hi = *reinterpret_cast<const float2 *>(d0 + i * kRS + 2);
          d[i][0] = lo.x; d[i][1] = lo.y; d[i][2] = hi.x; d[i][3] = hi.y;
        }
        const float *up = us + (4 * s + kq) * kKout + i16;
#pragma unroll
        for (int kg = 0; kg < KCH; ++kg)
#pragma unroll
          for (int q = 0; q < 16; ++q) u[kg][q] = up[q * kC * kKout + kg * kK];
      };
      auto mul_s = [&](bool first, const float (&d)[4][4], const float (&u)[KCH][16]) __attribute__((always_inline)) {
        // input transform V = Bt d B of the lane's patch; then the 16 point products:
        // A = V (block i16, channel kq), B = U (channel kq, filter i16)
        float t[4][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          t[0][j] = d[0][j] - d[2][j];
          t[1][j] = d[1][j] + d[2][j];
          t[2][j] = d[2][j] - d[1][j];
          t[3][j] = d[1][j] - d[3][j];
        }
        float V[16];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          V[4 * i + 0] = t[i][0] - t[i][2];
          V[4 * i + 1] = t[i][1] + t[i][2];
          V[4 * i + 2] = t[i][2] - t[i][1];
          V[4 * i + 3] = t[i][1] - t[i][3];
        }
#pragma unroll
        for (int q = 0; q < 16; ++q)
#pragma unroll
          for (int kg = 0; kg < KCH; ++kg)
            acc[kg][q] = __builtin_amdgcn_mfma_f32_16x16x4f32(V[q], u[kg][q], first ? zero : acc[kg][q], 0, 0, 0);
      };
      if constexpr (KCH == 2) {
        // Two filter groups: a quartet's transformed patch is used twice, 16 products per group.  The
        // filter fragments of a group are read into the registers whose products have just been
        // issued, one quartet ahead (u0: group 0, u1: group 1); the patch one quartet ahead as well.
        float u0[16], u1[16], V[16];
        auto read_d = [&](int s, float (&d)[4][4]) __attribute__((always_inline)) {
          const float *d0 = xs + (4 * s + kq) * kPS + (2 * tr) * kRS + 2 * i16;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float2 lo = *reinterpret_cast<const float2 *>(d0 + i * kRS);
            const float2 hi = *reinterpret_cast<const float2 *>(d0 + i * kRS + 2);
            d[i][0] = lo.x; d[i][1] = lo.y; d[i][2] = hi.x; d[i][3] = hi.y;
          }
        };
        auto read_u = [&](int s, int kg, float (&u)[16]) __attribute__((always_inline)) {
          const float *up = us + (4 * s + kq) * kKout + kg * kK + i16;
#pragma unroll
          for (int q = 0; q < 16; ++q) u[q] = up[q * kC * kKout];
        };
        auto xform = [&](const float (&d)[4][4]) __attribute__((always_inline)) {
          float t[4][4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            t[0][j] = d[0][j] - d[2][j];
            t[1][j] = d[1][j] + d[2][j];
            t[2][j] = d[2][j] - d[1][j];
            t[3][j] = d[1][j] - d[3][j];
          }
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            V[4 * i + 0] = t[i][0] - t[i][2];
            V[4 * i + 1] = t[i][1] + t[i][2];
            V[4 * i + 2] = t[i][2] - t[i][1];
            V[4 * i + 3] = t[i][1] - t[i][3];
          }
        };
        auto mul_g = [&](bool first, int kg, const float (&u)[16]) __attribute__((always_inline)) {
#pragma unroll
          for (int q = 0; q < 16; ++q) acc[kg][q] = __builtin_amdgcn_mfma_f32_16x16x4f32(V[q], u[q], first ? zero : acc[kg][q], 0, 0, 0);
        };
        read_d(0, dA);
        read_u(0, 0, u0);
        read_u(0, 1, u1);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const bool first = chunk == 0 && s == 0;
          __builtin_amdgcn_sched_barrier(0);
          xform(dA);
          __builtin_amdgcn_sched_barrier(0);
          if (s < 3) read_d(s + 1, dA);   // into the registers the transform has just consumed
          __builtin_amdgcn_sched_barrier(0);
          mul_g(first, 0, u0);
          __builtin_amdgcn_sched_barrier(0);
          if (s < 3) read_u(s + 1, 0, u0);
          __builtin_amdgcn_sched_barrier(0);
          mul_g(first, 1, u1);
          __builtin_amdgcn_sched_barrier(0);
          if (s < 3) read_u(s + 1, 1, u1);
        }
        __builtin_amdgcn_sched_barrier(0);
      } else {
      read_s(0, dA, uA);
      read_s(1, dB, uB);
      __builtin_amdgcn_sched_barrier(0);
      mul_s(chunk == 0, dA, uA);
      __builtin_amdgcn_sched_barrier(0);
      read_s(2, dA, uA);
      __builtin_amdgcn_sched_barrier(0);
      mul_s(false, dB, uB);
      __builtin_amdgcn_sched_barrier(0);
      read_s(3, dB, uB);
      __builtin_amdgcn_sched_barrier(0);
      mul_s(false, dA, uA);
      __builtin_amdgcn_sched_barrier(0);
      mul_s(false, dB, uB);
      __builtin_amdgcn_sched_barrier(0);
      }
    }
    }   // channel chunks
#pragma unroll
    for (int kg = 0; kg < KCH; ++kg) {
      // ---- output transform: lane holds blocks 4kq + v (v = 0..3) of filter (output channel) i16;
      // two blocks at a time keep few values alive
      float yv[4];
      unsigned char iv[4];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        float y00[2], y01[2], y10[2], y11[2];
#pragma unroll
        for (int w = 0; w < 2; ++w) {
          const int v = 2 * h + w;
          float sr[2][4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            sr[0][j] = acc[kg][j][v] + acc[kg][4 + j][v] + acc[kg][8 + j][v];
            sr[1][j] = acc[kg][4 + j][v] - acc[kg][8 + j][v] - acc[kg][12 + j][v];
          }
          y00[w] = sr[0][0] + sr[0][1] + sr[0][2]; y01[w] = sr[0][1] - sr[0][2] - sr[0][3];
          y10[w] = sr[1][0] + sr[1][1] + sr[1][2]; y11[w] = sr[1][1] - sr[1][2] - sr[1][3];
        }
        if constexpr (BWD) {
          // the blocks as they are: two rows of four consecutive columns per pair of blocks
          float *o0 = a.out + (((long)n * kKout + kg * kK + i16) * a.Hout + oy0 + 2 * tr) * a.Wout + ox0 + 8 * kq + 4 * h;
          *reinterpret_cast<float4 *>(o0) = make_float4(y00[0], y01[0], y00[1], y01[1]);
          *reinterpret_cast<float4 *>(o0 + a.Wout) = make_float4(y10[0], y11[0], y10[1], y11[1]);
        } else {
          // bias, ReLU, pooling: a block is one pooling window
#pragma unroll
          for (int w = 0; w < 2; ++w) {
            const int v = 2 * h + w;
            float m = y00[w];
            int arg = 0;
            if (y01[w] > m) { m = y01[w]; arg = 1; }
            if (y10[w] > m) { m = y10[w]; arg = 2; }
            if (y11[w] > m) { m = y11[w]; arg = 3; }
            const float o = m + bias[kg];
            yv[v] = o > 0.0f ? o : 0.0f;
            iv[v] = (unsigned char)(arg | (yv[v] > 0.0f ? 0 : kIdxInactive));
          }
        }
      }
      if constexpr (!BWD) {
        const long o = (((long)n * kKout + kg * kK + i16) * Hp + (oy0 >> 1) + tr) * Wp + (ox0 >> 1) + 4 * kq;
        *reinterpret_cast<float4 *>(a.out + o) = make_float4(yv[0], yv[1], yv[2], yv[3]);
        if (a.out_idx) *reinterpret_cast<uchar4 *>(a.out_idx + o) = make_uchar4(iv[0], iv[1], iv[2], iv[3]);
      }
    }
  }
}

inline bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

}  // namespace

// Forward: plain source tensor, 16 channels in and out, padded 3x3, ReLU + 2x2 pooling, whole 8 x 32
// tiles.  Backward-data of such a layer, or of one with 32 filters (two chunks of 16 source channels):
// pooled gradient + pooling bytes with the ReLU flags in, plain gradient out.
namespace {
bool wino_common(const ConvEngineArgs &a) {
  return (a.Cin == kC || a.Cin == 2 * kC) && (a.Kout == kK || a.Kout == 2 * kK) && a.R == 3 && a.S == 3 && a.pad_h == 1 && a.pad_w == 1 && !a.sample && !a.out_pool &&
         a.Hout == a.Hin && a.Wout == a.Win && a.Hout % 8 == 0 && a.Wout % 32 == 0 && aligned16(a.out) &&
         // the forward staging addresses the source with signed 32-bit BYTE offsets (negative = out of range)
         4L * a.N * a.Cin * a.Hin * a.Win < (1L << 31);
}
bool wino_is_bwd(const ConvEngineArgs &a) {
  return a.src_dz && a.w_flip && a.src_pool == 2 && a.src_act == ACT_RELU_FLAGGED && a.src_idx && a.act == ACT_IDENTITY &&
         a.pool == 1 && !a.bias && aligned16(a.src) && (reinterpret_cast<uintptr_t>(a.src_idx) & 3u) == 0;
}
}  // namespace
bool conv_wino_applies(const ConvEngineArgs &a) {
  if (!wino_common(a)) return false;
  if (wino_is_bwd(a)) return a.Kout == kK || a.Cin == 2 * kC;   // two filter groups: with two channel chunks only
  if (a.Cin != kC && a.Kout != 2 * kK) return false;   // forward, two channel chunks: with two filter groups only
  return !a.src_dz && !a.w_flip && a.act == ACT_RELU && a.pool == 2 && (!a.out_idx || (reinterpret_cast<uintptr_t>(a.out_idx) & 3u) == 0);
}

hipError_t launch_conv_wino(const ConvEngineArgs &a, hipStream_t stream) {
  if (!conv_wino_applies(a)) return hipErrorInvalidValue;
  WinoParams p;
  p.a = a;
  // 8-row tiles: three workgroups per CU instead of two (measured 80 vs 85 us on the 128 x 128 layer);
  // with two filter groups the accumulators take 128 registers and two workgroups stay resident
  const int grp = 1;
  p.tiles_x = a.Wout / 32;
  p.tiles_y = a.Hout / (8 * grp);
  p.items = a.N * p.tiles_x * p.tiles_y;
  const bool kk = a.Kout == 2 * kK;
  int blocks = chip().cus * ((grp == 2 || kk) ? 2 : 3);   // resident workgroups per CU (LDS, registers)
  if (blocks > p.items) blocks = p.items;
  p.xcd = blocks % 8 == 0;   // workgroups go to the eight XCDs in turn: see the kernel's tile loop
  const bool two = a.Cin == 2 * kC;
  if (wino_is_bwd(a)) {
    if (two && kk) hipLaunchKernelGGL((conv3x3_wino_kernel<1, true, 2, 2>), dim3(blocks), dim3(kWT), 0, stream, p);
    else if (two) hipLaunchKernelGGL((conv3x3_wino_kernel<1, true, 2, 1>), dim3(blocks), dim3(kWT), 0, stream, p);
    else hipLaunchKernelGGL((conv3x3_wino_kernel<1, true, 1, 1>), dim3(blocks), dim3(kWT), 0, stream, p);
  } else {
    if (kk && two) hipLaunchKernelGGL((conv3x3_wino_kernel<1, false, 2, 2>), dim3(blocks), dim3(kWT), 0, stream, p);
    else if (kk) hipLaunchKernelGGL((conv3x3_wino_kernel<1, false, 1, 2>), dim3(blocks), dim3(kWT), 0, stream, p);
    else hipLaunchKernelGGL((conv3x3_wino_kernel<1, false, 1, 1>), dim3(blocks), dim3(kWT), 0, stream, p);
  }
  return hipGetLastError();
}

}  // namespace dllk
