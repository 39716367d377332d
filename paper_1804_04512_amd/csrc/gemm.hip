// Dense-layer matrix products on fp32 MFMA (v_mfma_f32_16x16x4_f32), gfx950.
//
// Section II-A of the paper: the forward pass of a fully-connected layer over a minibatch is
// one matrix product, the backward pass one with the transposed weights, the gradient one
// more.  A single kernel serves all three through element strides:
//   C(m,n) = sum_k A(m,k) * B(k,n),   A(m,k) = A[m*a_m + k*a_k],  B(k,n) = B[k*b_k + n*b_n]
// with bias + activation, an optional act'(.) factor on the result (the data gradient leaves as
// dz of the layer below), split-K with a fixed-order second pass, and an optional in-place
// parameter update C_upd += step * C.
// Workgroup tile 128 x 64 x 32, four wavefronts of 64 x 32 each, register-prefetched k-tiles.
#include "dll_internal.h"
#include "small_bodies.h"

#include <type_traits>

namespace dllk {

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;
constexpr int BM = 128, BN = 64, BK = 32;
constexpr int LDK = 34;                // [x][k] layout (k-contiguous sources): row stride
constexpr int LDXA = 144, LDXB = 80;   // [k][x] layout (x-contiguous sources): row strides for 128 / 64 wide tiles
constexpr int A_TILE = BK * LDXA;      // 4608 floats >= BM * LDK
constexpr int B_TILE = BK * LDXB;      // 2560 floats >= BN * LDK

struct GemmParams {
  GemmArgs a;
  int k_per_split;   // multiple of BK
  int a_vec, b_vec;  // operand may be staged with 16-byte loads
  int c_vec;         // epilogue may use 16-byte accesses along n
};

__device__ __forceinline__ float act_apply(int act, float z) {
  if (act == ACT_SIGMOID) return 1.0f / (1.0f + expf(-z));
  if (act == ACT_RELU) return z > 0.0f ? z : 0.0f;
  return z;
}
__device__ __forceinline__ float act_deriv(int act, float out) {
  if (act == ACT_SIGMOID) return out * (1.0f - out);
  if (act == ACT_RELU) return out > 0.0f ? 1.0f : 0.0f;
  return 1.0f;
}

// One operand tile (XT along x, 32 along k) travels global -> registers -> LDS.  A thread
// carries groups of four elements that are neighbours along the source's contiguous axis:
// k-contiguous sources land in LDS as [x][34], x-contiguous ones as [k][XT+16]; both layouts
// give conflict-free MFMA operand reads.
template <int XT>
struct TileRegs {
  static constexpr int NV = XT * BK / 4 / kThreads;   // float4 per thread: 4 (XT = 128) or 2 (XT = 64)
  float4 v[NV];
  unsigned valid;   // generic loader: bit 4*it + e is set when element e of group `it` lies inside the operand
};

// Generic path: any strides, any alignment, ragged edges.  Every load is issued unconditionally
// from a clamped address (element 0 of the operand stands in for anything out of range) and the
// out-of-range elements are zeroed only when the tile is written to LDS: a load under a per-lane
// branch, or one whose value is touched right away, is waited for before the next one is issued,
// and a k-tile would cost as many memory round trips as it has groups.
template <int XT>
__device__ __forceinline__ void tile_load(TileRegs<XT> &t, const float *src, long sx, long sk, int x0, int k0, int X,
                                          int Kend, bool kcontig, bool vec) {
  constexpr int NV = TileRegs<XT>::NV;
  constexpr int TPR = XT / 4, RPP = kThreads / TPR;
  const int tid = threadIdx.x;
  const long stride = kcontig ? sk : sx;
  const int limit = kcontig ? Kend : X;
  long base[NV];
  int i0[NV];
  bool inr[NV];
#pragma unroll
  for (int it = 0; it < NV; ++it) {
    const int x = kcontig ? x0 + (tid >> 3) + 32 * it : x0 + 4 * (tid % TPR);
    const int k = kcontig ? k0 + 4 * (tid & 7) : k0 + (tid / TPR) + RPP * it;
    base[it] = (long)x * sx + (long)k * sk;
    i0[it] = kcontig ? k : x;
    inr[it] = kcontig ? x < X : k < Kend;
  }
  unsigned valid = 0;
  if (vec && (limit & 3) == 0) {   // uniform: whole aligned 16-byte groups, each entirely in or out of range
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const bool ok = inr[it] && i0[it] < limit;
      t.v[it] = *reinterpret_cast<const float4 *>(src + (ok ? base[it] : 0));
      valid |= ok ? (0xFu << (4 * it)) : 0u;
    }
  } else {
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      const bool e0 = inr[it] && i0[it] < limit, e1 = inr[it] && i0[it] + 1 < limit, e2 = inr[it] && i0[it] + 2 < limit,
                 e3 = inr[it] && i0[it] + 3 < limit;
      t.v[it].x = src[e0 ? base[it] : 0];
      t.v[it].y = src[e1 ? base[it] + stride : 0];
      t.v[it].z = src[e2 ? base[it] + 2 * stride : 0];
      t.v[it].w = src[e3 ? base[it] + 3 * stride : 0];
      valid |= ((e0 ? 1u : 0u) | (e1 ? 2u : 0u) | (e2 ? 4u : 0u) | (e3 ? 8u : 0u)) << (4 * it);
    }
  }
  t.valid = valid;
}

template <int XT>
__device__ __forceinline__ void tile_store(const TileRegs<XT> &t, float *dst, bool kcontig) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int it = 0; it < TileRegs<XT>::NV; ++it) {
    const unsigned m = t.valid >> (4 * it);
    const float4 v = make_float4((m & 1u) ? t.v[it].x : 0.f, (m & 2u) ? t.v[it].y : 0.f, (m & 4u) ? t.v[it].z : 0.f,
                                 (m & 8u) ? t.v[it].w : 0.f);
    if (kcontig) {
      float2 *d = reinterpret_cast<float2 *>(dst + ((tid >> 3) + 32 * it) * LDK + 4 * (tid & 7));
      d[0] = make_float2(v.x, v.y);
      d[1] = make_float2(v.z, v.w);
    } else {
      constexpr int TPR = XT / 4, RPP = kThreads / TPR;
      *reinterpret_cast<float4 *>(dst + ((tid / TPR) + RPP * it) * (XT + 16) + 4 * (tid % TPR)) = v;
    }
  }
}

// Workgroup tile 128 (m) x 64 (n) x 32 (k), four wavefronts of 64 x 32.  The n axis rides on
// the MFMA row axis, so a lane's four accumulator registers are four neighbouring columns of
// C and leave (or update the parameters) as one 16-byte access.  The next k-tile's global
// loads are in flight while the current one is multiplied (double-buffered LDS).
// FAST: both operands take the vector path (A_KC / B_KC say which axis is contiguous, A_OUT
// whether the act' factor is applied); otherwise the generic loader is used.
__global__ __launch_bounds__(kThreads, 2) void gemm_kernel(const GemmParams p) {
  __shared__ __attribute__((aligned(16))) float As[2][A_TILE];
  __shared__ __attribute__((aligned(16))) float Bs[2][B_TILE];
  const GemmArgs &a = p.a;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, kq = lane >> 4;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int kbeg = blockIdx.z * p.k_per_split;
  const int kend = min(a.Kdim, kbeg + p.k_per_split);
  const bool a_kc = a.a_k == 1, b_kc = a.b_k == 1;
  const int alx = a_kc ? LDK : 1, alk = a_kc ? 1 : LDXA;
  const int blx = b_kc ? LDK : 1, blk = b_kc ? 1 : LDXB;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 32;

  floatx4 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  // two register sets: tile t+2 is requested while tile t is multiplied and tile t+1 waits in
  // registers for its turn in LDS, so two k-tiles of global loads are always in flight
  TileRegs<BM> ta[2];
  TileRegs<BN> tb[2];
  auto load_tiles = [&](auto setc, int k0) {
    constexpr int S_ = decltype(setc)::value;
    tile_load<BM>(ta[S_], a.A, a.a_m, a.a_k, m0, k0, a.M, kend, a_kc, p.a_vec);
    tile_load<BN>(tb[S_], a.B, a.b_n, a.b_k, n0, k0, a.N, kend, b_kc, p.b_vec);
  };
  auto store_tiles = [&](auto setc, int buf) {
    constexpr int S_ = decltype(setc)::value;
    tile_store<BM>(ta[S_], As[buf], a_kc);
    tile_store<BN>(tb[S_], Bs[buf], b_kc);
  };
  // operand fragments are double-buffered in registers: the LDS reads of step s+1 are issued
  // before the MFMAs of step s (scheduling barriers keep that order)
  auto multiply = [&](int buf) {
    const float *Ab = As[buf] + (wm + i16) * alx + kq * alk;
    const float *Bb = Bs[buf] + (wn + i16) * blx + kq * blk;
    float af[2][4], bf[2][2];
    auto load_frags = [&](auto bc, int s) {
      constexpr int B_ = decltype(bc)::value;
#pragma unroll
      for (int i = 0; i < 4; ++i) af[B_][i] = Ab[i * 16 * alx + 4 * s * alk];
#pragma unroll
      for (int j = 0; j < 2; ++j) bf[B_][j] = Bb[j * 16 * blx + 4 * s * blk];
    };
    auto mfma_frags = [&](auto bc) {
      constexpr int B_ = decltype(bc)::value;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(bf[B_][j], af[B_][i], acc[i][j], 0, 0, 0);
    };
    load_frags(std::integral_constant<int, 0>{}, 0);
#pragma unroll
    for (int s = 0; s < BK / 4; s += 2) {
      load_frags(std::integral_constant<int, 1>{}, s + 1);
      __builtin_amdgcn_sched_barrier(0);
      mfma_frags(std::integral_constant<int, 0>{});
      __builtin_amdgcn_sched_barrier(0);
      if (s + 2 < BK / 4) load_frags(std::integral_constant<int, 0>{}, s + 2);
      __builtin_amdgcn_sched_barrier(0);
      mfma_frags(std::integral_constant<int, 1>{});
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;
  if (kbeg < kend) {
    load_tiles(S0{}, kbeg);
    if (kbeg + BK < kend) load_tiles(S1{}, kbeg + BK);
    store_tiles(S0{}, 0);
  }
  __syncthreads();
  for (int k0 = kbeg; k0 < kend; k0 += 2 * BK) {
    // LDS buffer 0 holds tile k0, register set 1 holds tile k0 + BK
    if (k0 + 2 * BK < kend) load_tiles(S0{}, k0 + 2 * BK);
    multiply(0);
    if (k0 + BK < kend) store_tiles(S1{}, 1);
    __syncthreads();
    if (k0 + BK >= kend) break;
    if (k0 + 3 * BK < kend) load_tiles(S1{}, k0 + 3 * BK);
    multiply(1);
    if (k0 + 2 * BK < kend) store_tiles(S0{}, 0);
    __syncthreads();
  }

  // fused parameter update: fetch the lane's eight 16-byte groups of the parameters with
  // unconditional loads from clamped addresses, so they are all in flight together
  float4 upd[4][2];
  if (a.update && p.c_vec && a.split_k == 1) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int m = m0 + wm + i * 16 + i16, n = n0 + wn + j * 16 + 4 * kq;
        const bool ok = m < a.M && n + 3 < a.N;
        upd[i][j] = *reinterpret_cast<const float4 *>(a.update + (ok ? (long)m * a.c_m + (long)n * a.c_n : 0));
      }
  }

  // lane holds C(m = i16, n = 4*kq + v) of each 16x16 tile; bias values and (per row) reference
  // outputs come in batches through clamped indices, never behind a per-element branch
  float bv[2][4];
  const bool direct = a.split_k == 1;
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int v = 0; v < 4; ++v) bv[j][v] = (direct && a.bias) ? a.bias[min(n0 + wn + j * 16 + 4 * kq + v, a.N - 1)] : 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + wm + i * 16 + i16;
    float rv[2][4];
    if (direct && a.C_ref) {
      const long om = (long)min(m, a.M - 1) * a.c_m;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) rv[j][v] = a.C_ref[om + (long)min(n0 + wn + j * 16 + 4 * kq + v, a.N - 1) * a.c_n];
    }
    // momentum: the row's two velocity groups, requested together from clamped addresses
    float4 velp[2];
    if (a.update && a.vel && p.c_vec && direct) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int n = n0 + wn + j * 16 + 4 * kq;
        const bool ok = m < a.M && n + 3 < a.N;
        velp[j] = *reinterpret_cast<const float4 *>(a.vel + (ok ? (long)m * a.c_m + (long)n * a.c_n : 0));
      }
    }
    if (m >= a.M) continue;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int n = n0 + wn + j * 16 + 4 * kq;
      if (n >= a.N) continue;
      float c[4] = {acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]};
      if (a.split_k > 1) {
        float *d = a.partial + ((long)blockIdx.z * a.M + m) * a.N + n;
        if (n + 3 < a.N && (a.N & 3) == 0) {
          *reinterpret_cast<float4 *>(d) = make_float4(c[0], c[1], c[2], c[3]);
        } else {
#pragma unroll
          for (int v = 0; v < 4; ++v)
            if (n + v < a.N) d[v] = c[v];
        }
        continue;
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) c[v] = act_apply(a.act, c[v] + bv[j][v]);
      const long o = (long)m * a.c_m + (long)n * a.c_n;
      if (a.C_ref) {
#pragma unroll
        for (int v = 0; v < 4; ++v) c[v] *= act_deriv(a.c_ref_act, rv[j][v]);
      }
      if (p.c_vec && n + 3 < a.N) {
        if (a.Cout) *reinterpret_cast<float4 *>(a.Cout + o) = make_float4(c[0], c[1], c[2], c[3]);
        if (a.update) {
          float4 u = upd[i][j];   // requested before the epilogue loop, all eight at once
          float4 vv = a.vel ? velp[j] : make_float4(0.f, 0.f, 0.f, 0.f);
          float *vp = a.vel ? &vv.x : nullptr;
          update_param(&u.x, vp, c[0], a.step, a.mu, a.decay); update_param(&u.y, vp ? vp + 1 : nullptr, c[1], a.step, a.mu, a.decay);
          update_param(&u.z, vp ? vp + 2 : nullptr, c[2], a.step, a.mu, a.decay); update_param(&u.w, vp ? vp + 3 : nullptr, c[3], a.step, a.mu, a.decay);
          *reinterpret_cast<float4 *>(a.update + o) = u;
          if (a.vel) *reinterpret_cast<float4 *>(a.vel + o) = vv;
        }
      } else {
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (n + v < a.N) {
            if (a.Cout) a.Cout[o + v * a.c_n] = c[v];
            if (a.update) update_param(a.update + o + v * a.c_n, a.vel ? a.vel + o + v * a.c_n : nullptr, c[v], a.step, a.mu, a.decay);
          }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------
// Persistent kernel for the vector-loadable case.  A unit of work is one (m-tile, n-tile,
// k-split); a workgroup walks units w, w+G, w+2G, ... and treats their k-tiles as ONE stream:
// the k-tile two places ahead is always in flight from global memory, also across unit
// boundaries, so neither the first loads of a unit nor (update mode) the parameter tile that
// the epilogue needs are waited for with the MFMA pipe idle.  Offsets are 32-bit byte
// offsets from the operand bases (the host checks the extents), one add per load.
// LDS holds k-contiguous sources as [x][34] and x-contiguous ones as [k][XT] with the x index
// XOR-ed by 16 on odd k: both give conflict-free operand reads, and two buffers of both
// operands stay under a third of the CU's LDS (three workgroups per CU).
constexpr int FA_TILE = BM * LDK;   // 4352 floats >= BK * BM
constexpr int FB_TILE = BN * LDK;   // 2176 floats >= BK * BN

template <int XT, bool KC>
struct SlotGeom {
  static constexpr int NV = XT * BK / 4 / kThreads;
  static constexpr int TPR = XT / 4, RPP = kThreads / TPR;
  __device__ static int xl(int tid, int it) { return KC ? (tid >> 3) + 32 * it : 4 * (tid % TPR); }
  __device__ static int kl(int tid, int it) { return KC ? 4 * (tid & 7) : (tid / TPR) + RPP * it; }
};

template <int XT, bool KC>
__device__ __forceinline__ void fast_tile_load(TileRegs<XT> &t, const float *src,
                                               const unsigned (&slot)[SlotGeom<XT, KC>::NV], unsigned sx, unsigned sk,
                                               int x0, int k0, int X, int Kend) {
  using G = SlotGeom<XT, KC>;
  const int tid = threadIdx.x;
  const unsigned base = 4u * ((unsigned)x0 * sx + (unsigned)k0 * sk);   // uniform
  const char *sb = reinterpret_cast<const char *>(src);
  float4 v[G::NV];
  if (x0 + XT <= X && k0 + BK <= Kend) {   // whole tile inside: plain loads
#pragma unroll
    for (int it = 0; it < G::NV; ++it) {
      const unsigned off = base + slot[it];
      v[it] = *reinterpret_cast<const float4 *>(sb + off);
    }
  } else {                                  // edge tile: clamped address, then select
    bool ok[G::NV];
#pragma unroll
    for (int it = 0; it < G::NV; ++it) {
      ok[it] = x0 + G::xl(tid, it) < X && k0 + G::kl(tid, it) < Kend;
      const unsigned off = ok[it] ? base + slot[it] : 0u;
      v[it] = *reinterpret_cast<const float4 *>(sb + off);
    }
#pragma unroll
    for (int it = 0; it < G::NV; ++it)
      if (!ok[it]) v[it] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
#pragma unroll
  for (int it = 0; it < G::NV; ++it) t.v[it] = v[it];
}

// LDS offset (in floats) of slot `it` of a thread: fixed for the whole kernel
template <int XT, bool KC>
__device__ __forceinline__ int fast_slot_lds(int tid, int it) {
  using G = SlotGeom<XT, KC>;
  const int x = G::xl(tid, it), k = G::kl(tid, it);
  return KC ? x * LDK + k : k * XT + (x ^ ((k & 1) << 4));
}

template <int XT, bool KC>
__device__ __forceinline__ void fast_tile_store(const TileRegs<XT> &t, float *dst, const int (&lds_off)[SlotGeom<XT, KC>::NV]) {
  using G = SlotGeom<XT, KC>;
#pragma unroll
  for (int it = 0; it < G::NV; ++it) {
    if (KC) {
      float2 *d = reinterpret_cast<float2 *>(dst + lds_off[it]);
      d[0] = make_float2(t.v[it].x, t.v[it].y);
      d[1] = make_float2(t.v[it].z, t.v[it].w);
    } else {
      *reinterpret_cast<float4 *>(dst + lds_off[it]) = t.v[it];
    }
  }
}

struct UnitPos {
  int unit;        // index of the (m-tile, n-tile, split) unit, or >= units when the stream has ended
  int kt, nkt;     // k-tile inside the unit, number of k-tiles of the unit
  int m0, n0, kbeg, kend, z;
  int second;      // pair launches: the unit belongs to the second product
};

// MODE fixes the epilogue at compile time (the launcher knows it), which keeps the code and the
// scalar state of the other forms out of the kernel:
//   0  split-K: the tile goes to the partial area as it is
//   1  fused parameter update, nothing else on the way (no bias, identity, no reference tensor);
//      the parameter tile is prefetched during the unit's last k-tile
//   2  everything else
// PAIR: one launch walks the units of TWO products of the same operand forms (p, then p2; both
// without split-K): a product too small to fill the chip rides along with a large one instead of
// paying for a launch of its own.
template <bool A_KC, bool B_KC, int MODE, bool PAIR>
__device__ __forceinline__ void gemm_fast_body(const GemmParams &p, const GemmParams &p2) {
  __shared__ __attribute__((aligned(16))) float As[2][FA_TILE];
  __shared__ __attribute__((aligned(16))) float Bs[2][FB_TILE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, kq = lane >> 4;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 32;
  const int tiles_n = (p.a.N + BN - 1) / BN, tiles_m = (p.a.M + BM - 1) / BM;
  const int units1 = tiles_m * tiles_n * p.a.split_k;
  const int tiles_n2 = PAIR ? (p2.a.N + BN - 1) / BN : 1;
  const int units = PAIR ? units1 + ((p2.a.M + BM - 1) / BM) * tiles_n2 : units1;
  auto args_of = [&](const UnitPos &u) __attribute__((always_inline)) -> const GemmArgs & { return (PAIR && u.second) ? p2.a : p.a; };

  auto locate = [&](UnitPos &u) __attribute__((always_inline)) {   // fills the fields that follow from u.unit
    if (u.unit >= units) return;
    if (PAIR && u.unit >= units1) {
      const int tile = u.unit - units1;
      u.second = 1;
      u.z = 0;
      u.m0 = (tile / tiles_n2) * BM;
      u.n0 = (tile % tiles_n2) * BN;
      u.kbeg = 0;
      u.kend = p2.a.Kdim;
    } else {
      const int tile = u.unit / p.a.split_k;
      u.second = 0;
      u.z = u.unit - tile * p.a.split_k;
      u.m0 = (tile / tiles_n) * BM;
      u.n0 = (tile % tiles_n) * BN;
      u.kbeg = u.z * p.k_per_split;
      u.kend = min(p.a.Kdim, u.kbeg + p.k_per_split);
    }
    u.nkt = max(1, (u.kend - u.kbeg + BK - 1) / BK);   // an empty split still writes its zero partial
    u.kt = 0;
  };
  auto advance = [&](UnitPos &u) __attribute__((always_inline)) {
    if (++u.kt < u.nkt) return;
    u.unit += gridDim.x;
    locate(u);
  };

  // per-slot byte offsets inside a tile (constant for a product; a pair launch works them out again
  // when its loading position crosses into the second product, once per workgroup)
  unsigned sa[SlotGeom<BM, A_KC>::NV], sb[SlotGeom<BN, B_KC>::NV];
  unsigned a_sx, a_sk, b_sx, b_sk;
  int slots_of = 0;
  auto slot_offsets = [&](const GemmArgs &a) __attribute__((always_inline)) {
    a_sx = (unsigned)a.a_m; a_sk = (unsigned)a.a_k; b_sx = (unsigned)a.b_n; b_sk = (unsigned)a.b_k;
#pragma unroll
    for (int it = 0; it < SlotGeom<BM, A_KC>::NV; ++it)
      sa[it] = 4u * ((unsigned)SlotGeom<BM, A_KC>::xl(tid, it) * a_sx + (unsigned)SlotGeom<BM, A_KC>::kl(tid, it) * a_sk);
#pragma unroll
    for (int it = 0; it < SlotGeom<BN, B_KC>::NV; ++it)
      sb[it] = 4u * ((unsigned)SlotGeom<BN, B_KC>::xl(tid, it) * b_sx + (unsigned)SlotGeom<BN, B_KC>::kl(tid, it) * b_sk);
  };
  slot_offsets(p.a);

  int la[SlotGeom<BM, A_KC>::NV], lb[SlotGeom<BN, B_KC>::NV];   // LDS offsets of the thread's slots
#pragma unroll
  for (int it = 0; it < SlotGeom<BM, A_KC>::NV; ++it) la[it] = fast_slot_lds<BM, A_KC>(tid, it);
#pragma unroll
  for (int it = 0; it < SlotGeom<BN, B_KC>::NV; ++it) lb[it] = fast_slot_lds<BN, B_KC>(tid, it);

  TileRegs<BM> ta[2];
  TileRegs<BN> tb[2];
  auto load_tiles = [&](auto setc, const UnitPos &u) __attribute__((always_inline)) {
    constexpr int S_ = decltype(setc)::value;
    const GemmArgs &a = args_of(u);
    if (PAIR && u.second != slots_of) { slot_offsets(a); slots_of = u.second; }
    const int k0 = u.kbeg + u.kt * BK;
    fast_tile_load<BM, A_KC>(ta[S_], a.A, sa, a_sx, a_sk, u.m0, k0, a.M, u.kend);
    fast_tile_load<BN, B_KC>(tb[S_], a.B, sb, b_sx, b_sk, u.n0, k0, a.N, u.kend);
  };
  auto store_tiles = [&](auto setc, int buf) __attribute__((always_inline)) {
    constexpr int S_ = decltype(setc)::value;
    fast_tile_store<BM, A_KC>(ta[S_], As[buf], la);
    fast_tile_store<BN, B_KC>(tb[S_], Bs[buf], lb);
  };

  // operand read pointers: fragment i of A sits 16*i rows (or columns) after the base; in the
  // swizzled layout lanes with odd k read even fragments 16 higher and odd ones 16 lower
  const int dsw = (kq & 1) << 4;
  const float *Ae = A_KC ? As[0] + (wm + i16) * LDK + kq : As[0] + kq * BM + wm + i16 + dsw;
  const float *Ao = A_KC ? Ae : As[0] + kq * BM + wm + i16 - dsw;
  const float *Be = B_KC ? Bs[0] + (wn + i16) * LDK + kq : Bs[0] + kq * BN + wn + i16 + dsw;
  const float *Bo = B_KC ? Be : Bs[0] + kq * BN + wn + i16 - dsw;
  constexpr int a_fx = A_KC ? 16 * LDK : 16, a_fk = A_KC ? 4 : 4 * BM;   // fragment and k-step strides
  constexpr int b_fx = B_KC ? 16 * LDK : 16, b_fk = B_KC ? 4 : 4 * BN;

  floatx4 acc[4][2];
  auto clear_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
  };
  clear_acc();

  auto multiply = [&](int buf) __attribute__((always_inline)) {
    const int ao = buf * FA_TILE, bo = buf * FB_TILE;
    float af[2][4], bf[2][2];
    auto load_frags = [&](auto bc, int s) __attribute__((always_inline)) {
      constexpr int B_ = decltype(bc)::value;
#pragma unroll
      for (int i = 0; i < 4; ++i) af[B_][i] = ((i & 1) ? Ao : Ae)[ao + i * a_fx + s * a_fk];
#pragma unroll
      for (int j = 0; j < 2; ++j) bf[B_][j] = ((j & 1) ? Bo : Be)[bo + j * b_fx + s * b_fk];
    };
    auto mfma_frags = [&](auto bc) __attribute__((always_inline)) {
      constexpr int B_ = decltype(bc)::value;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(bf[B_][j], af[B_][i], acc[i][j], 0, 0, 0);
    };
    load_frags(std::integral_constant<int, 0>{}, 0);
#pragma unroll
    for (int s = 0; s < BK / 4; s += 2) {
      load_frags(std::integral_constant<int, 1>{}, s + 1);
      __builtin_amdgcn_sched_barrier(0);
      mfma_frags(std::integral_constant<int, 0>{});
      __builtin_amdgcn_sched_barrier(0);
      if (s + 2 < BK / 4) load_frags(std::integral_constant<int, 0>{}, s + 2);
      __builtin_amdgcn_sched_barrier(0);
      mfma_frags(std::integral_constant<int, 1>{});
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // parameter tile of the unit whose last k-tile is about to be multiplied (update mode)
  constexpr bool upd_mode = MODE == 1;
  float4 upd[4][2];
  auto prefetch_update = [&](const UnitPos &u) __attribute__((always_inline)) {
    const GemmArgs &a = args_of(u);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int m = u.m0 + wm + i * 16 + i16, n = u.n0 + wn + j * 16 + 4 * kq;
        const bool ok = m < a.M && n + 3 < a.N;
        upd[i][j] = *reinterpret_cast<const float4 *>(a.update + (ok ? (long)m * a.c_m + (long)n * a.c_n : 0));
      }
  };

  // lane holds C(m = i16, n = 4*kq + v) of each 16x16 tile
  auto epilogue = [&](const UnitPos &u) __attribute__((always_inline)) {
    const GemmArgs &a = args_of(u);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = u.m0 + wm + i * 16 + i16;
      // momentum: the row's two velocity groups, requested together from clamped addresses
      float4 velp[2];
      if (MODE == 1 && a.vel) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int n = u.n0 + wn + j * 16 + 4 * kq;
          const bool ok = m < a.M && n + 3 < a.N;
          velp[j] = *reinterpret_cast<const float4 *>(a.vel + (ok ? (long)m * a.c_m + (long)n * a.c_n : 0));
        }
      }
      if (m >= a.M) continue;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int n = u.n0 + wn + j * 16 + 4 * kq;
        if (n >= a.N) continue;
        float c[4] = {acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]};
        if constexpr (MODE == 0) {
          float *d = a.partial + ((long)u.z * a.M + m) * a.N + n;
          if (n + 3 < a.N && (a.N & 3) == 0) {
            *reinterpret_cast<float4 *>(d) = make_float4(c[0], c[1], c[2], c[3]);
          } else {
#pragma unroll
            for (int v = 0; v < 4; ++v)
              if (n + v < a.N) d[v] = c[v];
          }
        } else if constexpr (MODE == 1) {
          const long o = (long)m * a.c_m + (long)n * a.c_n;
          if (n + 3 < a.N) {   // the launcher guarantees whole 16-byte groups (c_vec); a ragged last group falls through
            if (a.Cout) *reinterpret_cast<float4 *>(a.Cout + o) = make_float4(c[0], c[1], c[2], c[3]);
            float4 w4 = upd[i][j];
            if (a.vel) {
              float4 vv = velp[j];
              update_param(&w4.x, &vv.x, c[0], a.step, a.mu, a.decay); update_param(&w4.y, &vv.y, c[1], a.step, a.mu, a.decay);
              update_param(&w4.z, &vv.z, c[2], a.step, a.mu, a.decay); update_param(&w4.w, &vv.w, c[3], a.step, a.mu, a.decay);
              *reinterpret_cast<float4 *>(a.vel + o) = vv;
            } else {
              w4.x += a.step * c[0]; w4.y += a.step * c[1]; w4.z += a.step * c[2]; w4.w += a.step * c[3];
            }
            *reinterpret_cast<float4 *>(a.update + o) = w4;
          } else {
#pragma unroll
            for (int v = 0; v < 4; ++v)
              if (n + v < a.N) {
                if (a.Cout) a.Cout[o + v * a.c_n] = c[v];
                update_param(a.update + o + v * a.c_n, a.vel ? a.vel + o + v * a.c_n : nullptr, c[v], a.step, a.mu, a.decay);
              }
          }
        } else {
          // the group's bias values and reference outputs: eight loads issued together through clamped
          // 32-bit offsets from uniform bases (the launcher checks that C's extent fits), none of them
          // behind a per-element branch, which would make each wait for the one before
          float bv[4] = {0.0f, 0.0f, 0.0f, 0.0f}, rv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
          if (a.bias) {
#pragma unroll
            for (int v = 0; v < 4; ++v)
              bv[v] = *reinterpret_cast<const float *>(reinterpret_cast<const char *>(a.bias) + 4u * (unsigned)min(n + v, a.N - 1));
          }
          if (a.C_ref) {
            const unsigned om = (unsigned)m * (unsigned)a.c_m;
#pragma unroll
            for (int v = 0; v < 4; ++v)
              rv[v] = *reinterpret_cast<const float *>(reinterpret_cast<const char *>(a.C_ref) +
                                                       4u * (om + (unsigned)min(n + v, a.N - 1) * (unsigned)a.c_n));
          }
#pragma unroll
          for (int v = 0; v < 4; ++v) c[v] = act_apply(a.act, c[v] + bv[v]);
          const long o = (long)m * a.c_m + (long)n * a.c_n;
          if (a.C_ref) {
#pragma unroll
            for (int v = 0; v < 4; ++v) c[v] *= act_deriv(a.c_ref_act, rv[v]);
          }
          if (p.c_vec && n + 3 < a.N) {
            if (a.Cout) *reinterpret_cast<float4 *>(a.Cout + o) = make_float4(c[0], c[1], c[2], c[3]);
            if (a.update) {
              float4 w4 = *reinterpret_cast<const float4 *>(a.update + o);
              if (a.vel) {
                float4 vv = *reinterpret_cast<const float4 *>(a.vel + o);
                update_param(&w4.x, &vv.x, c[0], a.step, a.mu, a.decay); update_param(&w4.y, &vv.y, c[1], a.step, a.mu, a.decay);
                update_param(&w4.z, &vv.z, c[2], a.step, a.mu, a.decay); update_param(&w4.w, &vv.w, c[3], a.step, a.mu, a.decay);
                *reinterpret_cast<float4 *>(a.vel + o) = vv;
              } else {
                w4.x += a.step * c[0]; w4.y += a.step * c[1]; w4.z += a.step * c[2]; w4.w += a.step * c[3];
              }
              *reinterpret_cast<float4 *>(a.update + o) = w4;
            }
          } else {
#pragma unroll
            for (int v = 0; v < 4; ++v)
              if (n + v < a.N) {
                if (a.Cout) a.Cout[o + v * a.c_n] = c[v];
                if (a.update) update_param(a.update + o + v * a.c_n, a.vel ? a.vel + o + v * a.c_n : nullptr, c[v], a.step, a.mu, a.decay);
              }
          }
        }
      }
    }
  };

  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;
  UnitPos cur, ld;
  cur.unit = blockIdx.x;
  locate(cur);
  if (cur.unit >= units) return;
  ld = cur;
  load_tiles(S0{}, ld);
  advance(ld);
  if (ld.unit < units) { load_tiles(S1{}, ld); advance(ld); }
  store_tiles(S0{}, 0);
  __syncthreads();
  // one step: LDS buffer BUF holds the stream's current k-tile, register set 1-BUF the next one
  auto step = [&](auto bufc) __attribute__((always_inline)) -> bool {
    constexpr int BUF = decltype(bufc)::value;
    using SAME = std::integral_constant<int, BUF>;
    using OTHER = std::integral_constant<int, 1 - BUF>;
    const bool last_kt = cur.kt + 1 == cur.nkt;
    const bool more = !(last_kt && cur.unit + (int)gridDim.x >= units);   // a k-tile follows in the stream
    if (ld.unit < units) { load_tiles(SAME{}, ld); advance(ld); }         // two places ahead
    if constexpr (upd_mode) { if (last_kt) prefetch_update(cur); }
    multiply(BUF);
    if (more) store_tiles(OTHER{}, 1 - BUF);
    __syncthreads();
    if (last_kt) {
      epilogue(cur);
      clear_acc();
    }
    advance(cur);
    return more;
  };
  while (true) {
    if (!step(S0{})) break;
    if (!step(S1{})) break;
  }
}

template <bool A_KC, bool B_KC, int MODE>
__global__ __launch_bounds__(kThreads, 3) void gemm_fast_kernel(const GemmParams p) {
  gemm_fast_body<A_KC, B_KC, MODE, false>(p, p);
}
template <bool A_KC, bool B_KC>
__global__ __launch_bounds__(kThreads, 3) void gemm_fast_pair_kernel(const GemmParams p, const GemmParams p2) {
  gemm_fast_body<A_KC, B_KC, 1, true>(p, p2);
}

__global__ __launch_bounds__(kThreads) void gemm_splitk_reduce_kernel(const GemmArgs a) {
  const long total = (long)a.M * a.N;
  for (long e = (long)blockIdx.x * kThreads + threadIdx.x; e < total; e += (long)gridDim.x * kThreads) {
    const int m = (int)(e / a.N), n = (int)(e - (long)m * a.N);
    float c = 0.0f;
#pragma unroll 8
    for (int z = 0; z < a.split_k; ++z) c += a.partial[(long)z * total + e];
    if (a.bias) c += a.bias[n];
    c = act_apply(a.act, c);
    const long o = (long)m * a.c_m + (long)n * a.c_n;
    if (a.C_ref) c *= act_deriv(a.c_ref_act, a.C_ref[o]);
    if (a.Cout) a.Cout[o] = c;
    if (a.update) update_param(a.update + o, a.vel ? a.vel + o : nullptr, c, a.step, a.mu, a.decay);
  }
}

// The same for rows of whole 16-byte groups (N, c_m multiples of 4, c_n = 1, aligned bases): four
// neighbouring elements per thread, the loads of several splits in flight, additions in split order.
__global__ __launch_bounds__(kThreads) void gemm_splitk_reduce4_kernel(const GemmArgs a) {
  const long total = (long)a.M * a.N, groups = total / 4;
  for (long g = (long)blockIdx.x * kThreads + threadIdx.x; g < groups; g += (long)gridDim.x * kThreads) {
    const long e = 4 * g;
    const int m = (int)(e / a.N), n = (int)(e - (long)m * a.N);
    float c[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 8
    for (int z = 0; z < a.split_k; ++z) {
      const float4 v = *reinterpret_cast<const float4 *>(a.partial + (long)z * total + e);
      c[0] += v.x; c[1] += v.y; c[2] += v.z; c[3] += v.w;
    }
    const long o = (long)m * a.c_m + n;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      if (a.bias) c[v] += a.bias[n + v];
      c[v] = act_apply(a.act, c[v]);
      if (a.C_ref) c[v] *= act_deriv(a.c_ref_act, a.C_ref[o + v]);
    }
    if (a.Cout) *reinterpret_cast<float4 *>(a.Cout + o) = make_float4(c[0], c[1], c[2], c[3]);
    if (a.update) {
#pragma unroll
      for (int v = 0; v < 4; ++v) update_param(a.update + o + v, a.vel ? a.vel + o + v : nullptr, c[v], a.step, a.mu, a.decay);
    }
  }
}

__global__ __launch_bounds__(kThreads) void colsum_kernel(const float *A, int M, int N, float *out, float *update,
                                                         float step, float *vel, float mu) {
  colsum_block(A, M, N, out, update, step, vel, mu, blockIdx.x);
}

// One workgroup per sample: p = softmax(logits) with the row maximum subtracted,
// rowloss = -ln p[label], dlogits = (p - onehot) / B.  Rows of up to kRowCache classes are kept
// in LDS between the passes; longer rows are read back from `logits`.
constexpr int kRowCache = 4096;
__global__ __launch_bounds__(kThreads) void softmax_ce_kernel(float *logits, const int *labels, int B, int classes,
                                                             float *dlogits, float *rowloss, const float *partial,
                                                             int split_k, const float *bias) {
  __shared__ float sh[kThreads];
  __shared__ float cache[kRowCache];
  const int n = blockIdx.x, tid = threadIdx.x;
  float *row = logits + (long)n * classes;
  const bool cached = classes <= kRowCache;
  if (partial) {   // the product's split-K partials, added in split order, then the bias
    const long total = (long)B * classes;
    const float *p0 = partial + (long)n * classes;
    // four classes per thread and pass, four splits per round: sixteen loads are in flight
    // together, none of them behind a branch (a thread past the end of the row re-reads the last
    // class and drops the result); the additions keep the split order
    for (int j0 = tid; j0 < classes; j0 += 4 * kThreads) {
      int jq[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) jq[q] = min(j0 + q * kThreads, classes - 1);
      float c[4] = {0.0f, 0.0f, 0.0f, 0.0f};
      int z = 0;
      for (; z + 4 <= split_k; z += 4) {
        float v[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int q = 0; q < 4; ++q) v[u][q] = p0[(long)(z + u) * total + jq[q]];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int q = 0; q < 4; ++q) c[q] += v[u][q];
      }
      for (; z < split_k; ++z) {
        float v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = p0[(long)z * total + jq[q]];
#pragma unroll
        for (int q = 0; q < 4; ++q) c[q] += v[q];
      }
      float bq[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) bq[q] = bias ? bias[jq[q]] : 0.0f;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int j = j0 + q * kThreads;
        if (j < classes) {
          const float v = bias ? c[q] + bq[q] : c[q];
          row[j] = v;
          if (cached) cache[j] = v;
        }
      }
    }
  } else if (cached) {
    for (int j = tid; j < classes; j += kThreads) cache[j] = row[j];
  }
  __syncthreads();   // the row is complete (and visible to the whole workgroup) before it is read back
  const float *r = cached ? cache : row;
  float m = -INFINITY;
  for (int j = tid; j < classes; j += kThreads) m = fmaxf(m, r[j]);
  m = block_reduce(m, sh, true);
  float s = 0.0f;
  for (int j = tid; j < classes; j += kThreads) s += expf(r[j] - m);
  s = block_reduce(s, sh, false);
  const int label = labels[n];
  const float inv = 1.0f / s, invB = 1.0f / (float)B;
  for (int j = tid; j < classes; j += kThreads) {
    const float pj = expf(r[j] - m) * inv;
    dlogits[(long)n * classes + j] = (pj - (j == label ? 1.0f : 0.0f)) * invB;
  }
  if (tid == 0) rowloss[n] = -(r[label] - m - logf(s));
}

// One workgroup per sample: prob = softmax(logits) with the row maximum subtracted.
__global__ __launch_bounds__(kThreads) void softmax_prob_kernel(const float *logits, int classes, float *prob) {
  __shared__ float sh[kThreads];
  const int n = blockIdx.x, tid = threadIdx.x;
  const float *row = logits + (long)n * classes;
  float m = -INFINITY;
  for (int j = tid; j < classes; j += kThreads) m = fmaxf(m, row[j]);
  m = block_reduce(m, sh, true);
  float s = 0.0f;
  for (int j = tid; j < classes; j += kThreads) s += expf(row[j] - m);
  s = block_reduce(s, sh, false);
  const float inv = 1.0f / s;
  for (int j = tid; j < classes; j += kThreads) prob[(long)n * classes + j] = expf(row[j] - m) * inv;
}

__global__ __launch_bounds__(kThreads) void mean_kernel(const float *v, int count, float *out) { mean_block(v, count, out); }

constexpr int kStatBlocks = 32;

// scratch[ch][b] = sum over the block's slice of (v0 - v1); scratch[C*32 + ch*32 + b] = sum of squares
__global__ __launch_bounds__(kThreads) void visible_stats_kernel(const float *v0, const float *v1, int N, int C, int HW,
                                                                float *scratch) {
  __shared__ float sh[kThreads];
  const int ch = blockIdx.y, b = blockIdx.x;
  const long per = (long)N * HW;
  float s = 0.0f, q = 0.0f;
  for (long e = (long)b * kThreads + threadIdx.x; e < per; e += (long)kStatBlocks * kThreads) {
    const long nn = e / HW, r = e - nn * HW;
    const long o = (nn * C + ch) * HW + r;
    const float d = v0[o] - v1[o];
    s += d;
    q += d * d;
  }
  s = block_reduce(s, sh, false);
  q = block_reduce(q, sh, false);
  if (threadIdx.x == 0) {
    scratch[ch * kStatBlocks + b] = s;
    scratch[(C + ch) * kStatBlocks + b] = q;
  }
}

__global__ void visible_stats_final_kernel(const float *scratch, int N, int C, int HW, float scale, float *dc, float *mse,
                                           float *c_update, float step) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  double sq = 0.0;
  for (int ch = 0; ch < C; ++ch) {
    double s = 0.0;
    for (int b = 0; b < kStatBlocks; ++b) {
      s += (double)scratch[ch * kStatBlocks + b];
      sq += (double)scratch[(C + ch) * kStatBlocks + b];
    }
    const float g = (float)(s * (double)scale);
    if (dc) dc[ch] = g;
    if (c_update) c_update[ch] += step * g;
  }
  if (mse) *mse = (float)(sq / ((double)N * C * HW));
}

__global__ __launch_bounds__(kThreads) void copy_kernel(const float *src, float *dst, size_t count) {
  for (size_t e = (size_t)blockIdx.x * kThreads + threadIdx.x; e < count; e += (size_t)gridDim.x * kThreads) dst[e] = src[e];
}

}  // namespace

int gemm_pick_split_k(int M, int N, int Kdim) {
  if (gemm_is_small(M, N, Kdim)) return 1;   // the small-product kernel splits k inside the workgroup
  const long tiles = (long)((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  const int ksteps = (Kdim + BK - 1) / BK;
  int split = 1;
  while (tiles * split < 2L * chip().cus && split * 2 <= ksteps / 4 && split < 64) split *= 2;   // two units per compute unit
  return split;
}

namespace {

// What launch_gemm works out of a product before it picks a kernel.
struct GemmPlan {
  GemmParams p;
  dim3 grid;          // tiles along n, tiles along m, k splits
  bool a_kc, b_kc;    // operand is contiguous along k
  bool fast;          // the persistent vector kernel applies
  int mode;           // its epilogue form (see gemm_fast_body)
};

GemmPlan plan_gemm(const GemmArgs &a) {
  GemmPlan g;
  GemmParams &p = g.p;
  p.a = a;
  if (p.a.split_k < 1) p.a.split_k = 1;
  const int ksteps = (a.Kdim + BK - 1) / BK;
  p.k_per_split = ((ksteps + p.a.split_k - 1) / p.a.split_k) * BK;
  auto al16 = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
  // 16-byte loads need an aligned base and a leading stride of whole vectors
  p.a_vec = al16(a.A) && ((a.a_k == 1 ? a.a_m : a.a_k) % 4 == 0) && (a.a_k == 1 || a.a_m == 1);
  p.b_vec = al16(a.B) && ((a.b_k == 1 ? a.b_n : a.b_k) % 4 == 0) && (a.b_k == 1 || a.b_n == 1);
  p.c_vec = a.c_n == 1 && a.c_m % 4 == 0 && (!a.Cout || al16(a.Cout)) && (!a.update || al16(a.update)) && (!a.vel || al16(a.vel));
  g.grid = dim3((a.N + BN - 1) / BN, (a.M + BM - 1) / BM, p.a.split_k);
  // whole 16-byte groups along each operand's contiguous axis, the k ranges of the splits start
  // on multiples of 32, and every operand element lies within 4 GiB of its base (32-bit byte
  // offsets): then the persistent vector kernel runs, else the generic one
  g.a_kc = a.a_k == 1;
  g.b_kc = a.b_k == 1;
  const auto extent = [](long n0, long s0, long n1, long s1) { return 4 * ((n0 - 1) * s0 + (n1 - 1) * s1 + 4); };
  const bool small = extent(a.M, a.a_m, a.Kdim, a.a_k) < (1L << 32) && extent(a.N, a.b_n, a.Kdim, a.b_k) < (1L << 32) &&
                     extent(a.M, a.c_m, a.N, a.c_n) < (1L << 32) && a.a_m >= 0 && a.a_k >= 0 && a.b_n >= 0 && a.b_k >= 0 &&
                     a.c_m >= 0 && a.c_n >= 0;
  g.fast = small && p.a_vec && p.b_vec && (g.a_kc ? a.Kdim % 4 == 0 : a.M % 4 == 0) && (g.b_kc ? a.Kdim % 4 == 0 : a.N % 4 == 0);
  g.mode = p.a.split_k > 1 ? 0 : ((a.update && p.c_vec && !a.bias && a.act == ACT_IDENTITY && !a.C_ref) ? 1 : 2);
  return g;
}

}  // namespace

hipError_t launch_gemm(const GemmArgs &a, hipStream_t stream) {
  if (a.split_k <= 1 && (gemm_is_small(a.M, a.N, a.Kdim) || a.small_form)) return launch_gemm_small(a, stream);
  if (a.sm_labels) return hipErrorInvalidValue;   // the fused loss exists in the small-product kernel only
  const GemmPlan g = plan_gemm(a);
  const GemmParams &p = g.p;
  if (!g.fast) {
    hipLaunchKernelGGL(gemm_kernel, g.grid, dim3(kThreads), 0, stream, p);
  } else {
    const long units = (long)g.grid.x * g.grid.y * g.grid.z;
    const long resident = 3L * chip().cus;   // three resident workgroups per CU
    const dim3 pgrid((unsigned)(units < resident ? units : resident));
    const int mode = g.mode;
#define DLL_GEMM_LAUNCH(AK, BK_)                                                                                      \
  do {                                                                                                                 \
    if (mode == 0) hipLaunchKernelGGL((gemm_fast_kernel<AK, BK_, 0>), pgrid, dim3(kThreads), 0, stream, p);           \
    else if (mode == 1) hipLaunchKernelGGL((gemm_fast_kernel<AK, BK_, 1>), pgrid, dim3(kThreads), 0, stream, p);      \
    else hipLaunchKernelGGL((gemm_fast_kernel<AK, BK_, 2>), pgrid, dim3(kThreads), 0, stream, p);                     \
  } while (0)
    if (g.a_kc && g.b_kc) DLL_GEMM_LAUNCH(true, true);
    else if (g.a_kc && !g.b_kc) DLL_GEMM_LAUNCH(true, false);
    else if (!g.a_kc && g.b_kc) DLL_GEMM_LAUNCH(false, true);
    else DLL_GEMM_LAUNCH(false, false);
#undef DLL_GEMM_LAUNCH
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (p.a.split_k > 1 && !a.defer_reduce) {
    auto al16 = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
    const long total = (long)a.M * a.N;
    const bool vec = a.N % 4 == 0 && a.c_n == 1 && a.c_m % 4 == 0 && al16(a.partial) && (!a.Cout || al16(a.Cout));
    long blocks = ((vec ? total / 4 : total) + kThreads - 1) / kThreads;
    if (blocks > 2048) blocks = 2048;
    if (vec) hipLaunchKernelGGL(gemm_splitk_reduce4_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, p.a);
    else hipLaunchKernelGGL(gemm_splitk_reduce_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, p.a);
    e = hipGetLastError();
  }
  return e;
}

// Two independent products in one launch (the weight-gradient products of two dense layers: both
// update their parameters in place, neither reads what the other writes).  Where both take the
// persistent kernel's fused-update form with the same operand forms, the units of the second are
// appended to the first's; else they are launched one after the other.
hipError_t launch_gemm_pair(const GemmArgs &a, const GemmArgs &b, hipStream_t stream) {
  const bool a_small = a.split_k <= 1 && gemm_is_small(a.M, a.N, a.Kdim), b_small = b.split_k <= 1 && gemm_is_small(b.M, b.N, b.Kdim);
  if (!a_small && !b_small && !a.sm_labels && !b.sm_labels && a.split_k <= 1 && b.split_k <= 1) {
    const GemmPlan ga = plan_gemm(a), gb = plan_gemm(b);
    if (ga.fast && gb.fast && ga.mode == 1 && gb.mode == 1 && ga.a_kc == gb.a_kc && ga.b_kc == gb.b_kc) {
      const long units = (long)ga.grid.x * ga.grid.y + (long)gb.grid.x * gb.grid.y;
      const long resident = 3L * chip().cus;
      const dim3 pgrid((unsigned)(units < resident ? units : resident));
      if (ga.a_kc && ga.b_kc) hipLaunchKernelGGL((gemm_fast_pair_kernel<true, true>), pgrid, dim3(kThreads), 0, stream, ga.p, gb.p);
      else if (ga.a_kc) hipLaunchKernelGGL((gemm_fast_pair_kernel<true, false>), pgrid, dim3(kThreads), 0, stream, ga.p, gb.p);
      else if (ga.b_kc) hipLaunchKernelGGL((gemm_fast_pair_kernel<false, true>), pgrid, dim3(kThreads), 0, stream, ga.p, gb.p);
      else hipLaunchKernelGGL((gemm_fast_pair_kernel<false, false>), pgrid, dim3(kThreads), 0, stream, ga.p, gb.p);
      return hipGetLastError();
    }
  }
  const hipError_t e = launch_gemm(a, stream);
  return e != hipSuccess ? e : launch_gemm(b, stream);
}

hipError_t launch_colsum(const float *A, int M, int N, float *out, float *update, float step, float *vel, float mu,
                         hipStream_t stream) {
  hipLaunchKernelGGL(colsum_kernel, dim3((N + kColsumCols - 1) / kColsumCols), dim3(kThreads), 0, stream, A, M, N, out, update,
                     step, vel, mu);
  return hipGetLastError();
}

hipError_t launch_softmax_ce(float *logits, const int *labels, int B, int classes, float *loss, float *dlogits,
                             float *rowloss, const float *partial, int split_k, const float *bias, hipStream_t stream) {
  hipLaunchKernelGGL(softmax_ce_kernel, dim3(B), dim3(kThreads), 0, stream, logits, labels, B, classes, dlogits, rowloss,
                     partial, split_k, bias);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (!loss) return e;   // the caller takes the mean of rowloss later (step closing kernel)
  hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(kThreads), 0, stream, rowloss, B, loss);
  return hipGetLastError();
}

hipError_t launch_softmax_prob(const float *logits, int B, int classes, float *prob, hipStream_t stream) {
  hipLaunchKernelGGL(softmax_prob_kernel, dim3(B), dim3(kThreads), 0, stream, logits, classes, prob);
  return hipGetLastError();
}

size_t visible_stats_scratch_floats(int, int C, int) { return (size_t)2 * C * kStatBlocks; }

hipError_t launch_visible_stats(const float *v0, const float *v1, int N, int C, int HW, float scale, float *dc, float *mse,
                                float *c_update, float step, float *scratch, hipStream_t stream) {
  hipLaunchKernelGGL(visible_stats_kernel, dim3(kStatBlocks, C), dim3(kThreads), 0, stream, v0, v1, N, C, HW, scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(visible_stats_final_kernel, dim3(1), dim3(64), 0, stream, scratch, N, C, HW, scale, dc, mse, c_update,
                     step);
  return hipGetLastError();
}

hipError_t launch_copy(const float *src, float *dst, size_t count, hipStream_t stream) {
  size_t blocks = (count + kThreads - 1) / kThreads;
  if (blocks > 4096) blocks = 4096;
  if (blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, src, dst, count);
  return hipGetLastError();
}

}  // namespace dllk
