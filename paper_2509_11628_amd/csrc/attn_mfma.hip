// bf16 MFMA attention for gfx950: softmax(q k^T / sqrt(hd)) v without mask, online softmax
// in fp32 (no T x T matrix is ever written).
//
// One block = 128 queries of one (row, head): 4 waves x 32 queries.  Keys/values stream
// through LDS in tiles of 64 keys, double buffered, one barrier per tile.
// Both contractions run on v_mfma_f32_32x32x16_bf16 producing TRANSPOSED tiles:
//   S^T[key][query] = K q^T   (A operand = key rows from LDS, B operand = the wave's query
//                              rows, held in registers for the whole kernel)
//   O^T[d][query]  += V^T P^T (A operand = V^T from LDS, B operand = P^T)
// In both results a lane's 16 values belong to ONE query (column lane % 32), so the softmax
// statistics and the rescaling of O are lane-local; only the max/sum over the lane pair
// (lane, lane ^ 32) needs a shuffle.  The P^T operand is taken straight from the S^T
// accumulators: the MFMA reduction index is a dummy, so the keys are simply fed to the second
// MFMA in the order the first one left them in the lane (keys 16t+4h+0..3, 16t+8+4h+0..3 for
// half-wave h), and V^T is read from LDS in that same order.
// V is transposed on its way into LDS (register transposes of 4-key x 8-dim blocks) into a swizzled,
// key-permuted layout.
// Three kernels: a tiled one (keys/values in 64-key tiles staged through registers, online softmax); for
// head_dim 128 a tiled one whose tiles go global -> LDS directly and whose V^T fragments come from the
// transposing LDS read (no staging, no register transposes; the next tile's scores are issued under the
// current tile's softmax); and, for T <= 256, one that holds the whole sequence of a head in LDS and takes
// the softmax in one pass.
// head_dim is padded with zeros to a multiple of 16 for q k^T and of 32 for P V.
#include <type_traits>

#include "gemm.h"

namespace speca {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

union Frag {
  uint4 u;
  bf16x8 v;
};

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// two floats -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ inline uint32_t cvt_pk_bf16(float a, float b) {
  const floatx2 f = {a, b};
  const bf16x2 r = __builtin_convertvector(f, bf16x2);
  return *reinterpret_cast<const uint32_t*>(&r);
}

// 2^x by the hardware instruction alone (inputs are <= 0 here; results below the normal range flush
// to 0, -inf gives 0): exp2f() wraps it in range checks and a rescale, ~5 vector instructions per value.
__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Transposed value tile in LDS: row = head dimension d, NK keys per row, rows unpadded.  The second
// MFMA wants, per lane and 16-key step t, the keys 16t + 4h + {0..3} and 16t + 8 + 4h + {0..3}
// (h = lane / 32): the keys of every group of 16 are stored in the order [0-3, 8-11 | 4-7, 12-15], so
// each half-wave's eight keys are ONE 16-byte chunk (chunk 2t + h) and a fragment is one
// ds_read_b128.  The chunk position is XOR-swizzled with the row so that the 16 lanes of a read
// phase (16 consecutive rows, same chunk) cover all 64 banks: with 64-key rows (32 words) the row
// parity supplies one bank bit and d & 7 the other three; with 256-key rows (a multiple of 64 words)
// all four come from d & 15.  The higher bits of d are XORed in as well: the transposing writer's
// lanes hold rows 8 apart (same d & 7), and without them its 8-byte writes would pile 8-deep onto two
// bank groups; with them they are at most 2-deep (checked by enumeration for head_dim 64 / 128).
// (Padded rows with two 8-byte reads per fragment measured 58 % of the LDS-active cycles as
// bank-conflict stalls.)
template <int NK>
__device__ inline int vt_swz(int d) {
  return NK % 128 == 0 ? ((d & 15) ^ ((d >> 4) & 7)) : ((d & 7) ^ ((d >> 3) & 7));
}
// element offset of the chunk that holds keys [16t + 4h .. ] u [16t + 8 + 4h ..] of dimension d
template <int NK>
__device__ inline int vt_read_off(int d, int t, int h) {
  return d * NK + (((2 * t + h) ^ vt_swz<NK>(d)) << 3);
}
// element offsets where the keys 8kb .. 8kb+3 (lo) and 8kb+4 .. 8kb+7 (hi) of dimension d go (8 bytes each)
template <int NK>
__device__ inline void vt_write_off(int d, int kb, int* lo, int* hi) {
  const int c = 2 * (kb >> 1), half = kb & 1, sw = vt_swz<NK>(d);
  *lo = d * NK + ((c ^ sw) << 3) + 4 * half;
  *hi = d * NK + (((c + 1) ^ sw) << 3) + 4 * half;
}

// Tiled kernel (T > 256): per 64-key tile, load the next tile into registers, compute the current one
// from LDS (S^T, softmax, O^T), store the next tile to LDS, one barrier.  Registers are capped so that
// two blocks share a CU (two waves per SIMD): the exponentials and conversions of one wave overlap
// the MFMAs of the other.  A software-pipelined variant that issued S of tile k+1 before the softmax
// of tile k needed > 256 registers (one wave per SIMD, accumulators shuttled through AGPRs: 190
// register moves per tile) and measured 455 / 596 TFLOP/s at 4608 / 27 286 tokens against 565 / 741.
template <int HD>
__global__ __launch_bounds__(256, 2) void attention_mfma_kernel(const uint16_t* __restrict__ qkv, uint16_t* __restrict__ out, int64_t ldo,
                                                             int T, int H, float scale_log2e) {
  constexpr int HD16 = (HD + 15) / 16 * 16, HD32 = (HD + 31) / 32 * 32;
  constexpr int KS = HD16 / 16;         // reduction steps of q k^T
  constexpr int DT = HD32 / 32;         // 32-row tiles of O^T
  constexpr int KST = HD16 + 8;         // LDS row stride of the key tile (elements)
  constexpr int VTILE = HD32 * 64;      // elements of one transposed value tile (see vt_read_off)
  constexpr int CH = HD / 8;            // 16-byte chunks per key/value row
  constexpr int K_CHUNKS = (64 * CH + 255) / 256;
  static_assert(HD % 8 == 0, "head_dim must be a multiple of 8");
  extern __shared__ __align__(16) uint16_t smem[];
  uint16_t* Ks = smem;                        // [2][64][KST]
  uint16_t* Vt = smem + 2 * 64 * KST;         // [2][VTILE]

  const int row = blockIdx.z, head = blockIdx.y, q0 = blockIdx.x * 128;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int64_t D = static_cast<int64_t>(H) * HD;
  const uint16_t* base = qkv + static_cast<int64_t>(row) * T * 3 * D + head * HD;

  // zero padding of both buffers: key columns [HD, HD16) and value rows [HD, HD32); never overwritten
  if (HD16 > HD)
    for (int i = tid; i < 2 * 64 * (HD16 - HD); i += 256) Ks[(i / (HD16 - HD)) * KST + HD + i % (HD16 - HD)] = 0;
  if (HD32 > HD)
    for (int i = tid; i < 2 * (HD32 - HD) * 64; i += 256) {
      const int b = i / ((HD32 - HD) * 64), r = (i / 64) % (HD32 - HD), c = i % 64;
      Vt[b * VTILE + (HD + r) * 64 + c] = 0;      // whole rows: the order inside a row does not matter
    }

  // the wave's 32 queries as B operand, resident in registers
  Frag qf[KS];
  {
    const int q = q0 + wave * 32 + l32;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int d = ks * 16 + lhi * 8;
      qf[ks].u = (q < T && d < HD) ? *reinterpret_cast<const uint4*>(base + static_cast<int64_t>(q) * 3 * D + d) : make_uint4(0, 0, 0, 0);
    }
  }

  floatx16 o[DT];
#pragma unroll
  for (int i = 0; i < DT; ++i)
#pragma unroll
    for (int q = 0; q < 16; ++q) o[i][q] = 0.0f;
  float mrun = -INFINITY, lrun = 0.0f;     // running max of the raw scores and this lane's partial sum

  uint4 rk[K_CHUNKS], rv[4];
  const bool v_thread = tid < 16 * CH;          // 4 keys x 8 dims per thread
  // The 4-key blocks are numbered so that the two blocks a 32-lane write phase touches differ in the
  // half of the 16-byte chunk they fill (2-deep bank conflicts at most).
  const int v_a = tid / CH, v_dc = tid % CH;
  const int v_k4 = (v_a & ~3) | ((v_a & 1) << 1) | ((v_a >> 1) & 1);
  auto load_global = [&](int k0) {
#pragma unroll
    for (int c = 0; c < K_CHUNKS; ++c) {
      const int id = tid + c * 256;
      const int key = id / CH, dc = id - key * CH;
      rk[c] = (id < 64 * CH && k0 + key < T) ? *reinterpret_cast<const uint4*>(base + static_cast<int64_t>(k0 + key) * 3 * D + D + dc * 8)
                                             : make_uint4(0, 0, 0, 0);
    }
    if (v_thread) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int key = k0 + v_k4 * 4 + i;
        rv[i] = key < T ? *reinterpret_cast<const uint4*>(base + static_cast<int64_t>(key) * 3 * D + 2 * D + v_dc * 8) : make_uint4(0, 0, 0, 0);
      }
    }
  };
  auto store_lds = [&](int buf) {
#pragma unroll
    for (int c = 0; c < K_CHUNKS; ++c) {
      const int id = tid + c * 256;
      const int key = id / CH, dc = id - key * CH;
      if (id < 64 * CH) *reinterpret_cast<uint4*>(Ks + (buf * 64 + key) * KST + dc * 8) = rk[c];
    }
    if (v_thread) {
      // rv[i] = 8 dims of key i  ->  8 rows (dims) of 4 keys
      const uint32_t w[4][4] = {{rv[0].x, rv[0].y, rv[0].z, rv[0].w}, {rv[1].x, rv[1].y, rv[1].z, rv[1].w},
                                {rv[2].x, rv[2].y, rv[2].z, rv[2].w}, {rv[3].x, rv[3].y, rv[3].z, rv[3].w}};
      const int c_ = 2 * (v_k4 >> 2) + (v_k4 & 1), h_ = (v_k4 >> 1) & 1;
#pragma unroll
      for (int dd = 0; dd < 8; ++dd) {
        const int d_ = v_dc * 8 + dd;
        uint32_t r[2];
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          const uint32_t a = w[2 * kk][dd >> 1], b = w[2 * kk + 1][dd >> 1];
          r[kk] = (dd & 1) ? ((a >> 16) | (b & 0xFFFF0000u)) : ((a & 0xFFFFu) | (b << 16));
        }
        *reinterpret_cast<uint2*>(Vt + buf * VTILE + d_ * 64 + ((c_ ^ vt_swz<64>(d_)) << 3) + 4 * h_) = make_uint2(r[0], r[1]);
      }
    }
  };

  const int ntiles = (T + 63) / 64;
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt < ntiles; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < ntiles) load_global((kt + 1) * 64);

    // S^T for the two 32-key sub-tiles
    floatx16 s[2];
#pragma unroll
    for (int st = 0; st < 2; ++st) {
#pragma unroll
      for (int q = 0; q < 16; ++q) s[st][q] = 0.0f;
      const uint16_t* kp = Ks + (buf * 64 + st * 32 + l32) * KST + lhi * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        Frag kf;
        kf.u = *reinterpret_cast<const uint4*>(kp + ks * 16);
        s[st] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf.v, qf[ks].v, s[st], 0, 0, 0);
      }
    }
    // mask the ragged tail (last tile only), row max of the raw scores over the lane pair
    const int kbase = kt * 64;
    if (kbase + 64 > T) {
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int q = 0; q < 16; ++q) {
          const int key = kbase + st * 32 + 8 * (q >> 2) + 4 * lhi + (q & 3);
          if (key >= T) s[st][q] = -INFINITY;
        }
    }
    float tmax = -INFINITY;
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int q = 0; q < 16; ++q) tmax = fmaxf(tmax, s[st][q]);
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    // mrun is the running maximum of the RAW scores; the scale (> 0) and log2(e) enter in one fma per score
    const float mnew = fmaxf(mrun, tmax);
    const float moff = mnew * scale_log2e;
    float psum = 0.0f;
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const float p = fast_exp2(fmaf(s[st][q], scale_log2e, -moff));
        s[st][q] = p;
        psum += p;
      }
    if (__any(mnew != mrun)) {       // the running maximum moved somewhere in the wave: rescale (rare after the first tiles)
      const float corr = fast_exp2(mrun * scale_log2e - moff);
      lrun *= corr;
#pragma unroll
      for (int i = 0; i < DT; ++i)
#pragma unroll
        for (int q = 0; q < 16; ++q) o[i][q] *= corr;
      mrun = mnew;
    }
    lrun += psum;

    // O^T += V^T P^T, four reduction steps of 16 keys
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int st = t >> 1, j0 = (t & 1) * 8;      // accumulator entries j0 .. j0+7 of sub-tile st
      Frag pf;
      pf.u = make_uint4(cvt_pk_bf16(s[st][j0], s[st][j0 + 1]), cvt_pk_bf16(s[st][j0 + 2], s[st][j0 + 3]),
                        cvt_pk_bf16(s[st][j0 + 4], s[st][j0 + 5]), cvt_pk_bf16(s[st][j0 + 6], s[st][j0 + 7]));
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        Frag vf;
        vf.u = *reinterpret_cast<const uint4*>(Vt + buf * VTILE + vt_read_off<64>(dt * 32 + l32, t, lhi));
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf.v, o[dt], 0, 0, 0);
      }
    }
    if (kt + 1 < ntiles) store_lds(buf ^ 1);
    __syncthreads();
  }

  const float ltot = lrun + __shfl_xor(lrun, 32, 64);
  const float inv = 1.0f / ltot;
  const int q = q0 + wave * 32 + l32;
  if (q < T) {
    uint16_t* op = out + (static_cast<int64_t>(row) * T + q) * ldo + head * HD;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int d = dt * 32 + 8 * jj + 4 * lhi;
        if (d < HD) {
          uint2 r;
          r.x = cvt_pk_bf16(o[dt][4 * jj] * inv, o[dt][4 * jj + 1] * inv);
          r.y = cvt_pk_bf16(o[dt][4 * jj + 2] * inv, o[dt][4 * jj + 3] * inv);
          *reinterpret_cast<uint2*>(op + d) = r;
        }
      }
  }
}

// ---------------------------------------------------------------------------------------------
// Tiled kernel for head_dim 128 whose key and value tiles go global -> LDS directly
// (global_load_lds_dwordx4: lane l's 16 bytes land at the wave-uniform LDS address + 16 l) and whose
// V^T operand is formed by the transposing LDS read, so nothing is staged or transposed in registers.
//
// Both tiles are stored row-major as they are in memory: 64 keys x 256 bytes (16 chunks of 16 bytes).
// One load instruction covers 4 rows; lane l supplies the chunk stored at position l % 16 of row l / 16.
// Keys:   S^T = K q^T reads, per lane, chunk 2 ks + h of row l32 (ds_read_b128); chunk c of row r sits at
//         position c ^ (r & 15), so the 16 lanes of a read phase touch all 64 banks once.
// Values: ds_read_b64_tr_b16, per group of 16 lanes: lane j points at 4 consecutive dims
//         d0 + 4 (j % 4) of key k0 + j / 4, and lane i of the group receives dim d0 + i of the keys
//         k0 .. k0 + 3 (measured lane layout).  Two such reads (keys 16 t + 4 h + 0..3 and
//         16 t + 8 + 4 h + 0..3) are one A fragment of V^T in exactly the key order the S^T
//         accumulators hand P^T to the second MFMA.  The four rows a half-wave reads are moved to
//         different 64-byte bank groups: chunk c of row r sits at position
//         c ^ (4 (r & 3) + ((r >> 2) & 3)).
// Rows beyond T are read from row T - 1 (valid memory): their scores are masked to -inf, so their
// probabilities are exactly 0 and the finite values they multiply do not matter.
// Ring: two buffers; per tile the waves wait for their own loads with vmcnt(0) (the only safe wait
// for these loads), one barrier, loads of the next tile are issued into the buffer just freed.
#define SPECA_ATTN_GLL(src, dst)                                                                                  \
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src),                         \
                                   (__attribute__((address_space(3))) void*)(dst), 16, 0, 0)
typedef short short4v __attribute__((ext_vector_type(4)));

template <bool PIPE>
__global__ __launch_bounds__(256, 2) void attention_dma_kernel(const uint16_t* __restrict__ qkv, uint16_t* __restrict__ out, int64_t ldo,
                                                            int T, int H, float scale_log2e) {
  constexpr int HD = 128, KS = 8, DT = 4;
  constexpr int TILE = 64 * HD;               // elements of one key or value tile
  extern __shared__ __align__(16) uint16_t smem[];
  uint16_t* Ks = smem;                        // [2][64][128]
  uint16_t* Vs = smem + 2 * TILE;             // [2][64][128]

  const int row = blockIdx.z, head = blockIdx.y, q0 = blockIdx.x * 128;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int64_t D = static_cast<int64_t>(H) * HD;
  const uint16_t* base = qkv + static_cast<int64_t>(row) * T * 3 * D + head * HD;

  Frag qf[KS];
  {
    const int q = q0 + wave * 32 + l32;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qf[ks].u = q < T ? *reinterpret_cast<const uint4*>(base + static_cast<int64_t>(q) * 3 * D + ks * 16 + lhi * 8) : make_uint4(0, 0, 0, 0);
  }
  floatx16 o[DT];
#pragma unroll
  for (int i = 0; i < DT; ++i)
#pragma unroll
    for (int q = 0; q < 16; ++q) o[i][q] = 0.0f;
  float mrun = -INFINITY, lrun = 0.0f;

  // loader: wave w issues instructions i = w, w + 4, w + 8, w + 12 of each tile (16 per tile, 4 rows each);
  // lane -> row 4 i + lane / 16, stored position lane % 16
  const int lr = lane >> 4, lp = lane & 15;
  // The source chunk of a lane does not depend on the instruction (rows 4 i + lr with i = wave + 4 g: r & 15 and
  // the value swizzle only see 4 wave + lr), so a tile's addresses are one per-lane 32-bit offset on top of a
  // wave-uniform row pointer: no per-load vector arithmetic.  Only a ragged last tile clamps rows per lane.
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int row3d = static_cast<int>(3 * D);
  const int koff = lr * row3d + static_cast<int>(D) + ((lp ^ ((4 * wave_u + lr) & 15)) << 3);
  const int voff = lr * row3d + 2 * static_cast<int>(D) + ((lp ^ (4 * lr + (wave_u & 3))) << 3);
  auto issue = [&](int k0, int buf, uint16_t* dst, int off) {
    if (k0 + 64 <= T) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int i = wave_u + 4 * g;
        const uint16_t* ub = base + static_cast<int64_t>(k0 + 4 * i) * row3d;      // wave-uniform
        SPECA_ATTN_GLL(ub + off, dst + buf * TILE + i * 512);
      }
    } else {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int i = wave_u + 4 * g;
        int key = k0 + 4 * i + lr;
        key = key < T ? key : T - 1;
        SPECA_ATTN_GLL(base + static_cast<int64_t>(key) * row3d + (off - lr * row3d), dst + buf * TILE + i * 512);
      }
    }
  };
  auto issue_k = [&](int k0, int buf) { issue(k0, buf, Ks, koff); };
  auto issue_v = [&](int k0, int buf) { issue(k0, buf, Vs, voff); };
  const int kpos_sw = l32 & 15;               // key row l32 (+32): r & 15
  // value reader: 16-lane group g = lane / 16, j = lane % 16: key k0 + j / 4 with k0 = 16 t + 4 (g >> 1) (+ 8),
  // dims dt * 32 + 16 (g & 1) + 4 (j % 4) .. + 3: chunk dt * 4 + 2 (g & 1) + (j % 4) / 2, half (j % 2)
  const int vg = lane >> 4, vj = lane & 15;
  const int vkey0 = 4 * (vg >> 1) + (vj >> 2);                     // key inside the 16-key step, first read (second: + 8)
  const int vchunk0 = 2 * (vg & 1) + ((vj & 3) >> 1);              // chunk inside the 32-dim block
  const int vhalf = (vj & 1) * 4;                                  // element offset inside the chunk

  // S^T of the 64 keys in key buffer kb
  auto scores = [&](floatx16 (&s)[2], int kb) {
#pragma unroll
    for (int st = 0; st < 2; ++st) {
#pragma unroll
      for (int q = 0; q < 16; ++q) s[st][q] = 0.0f;
      const uint16_t* kp = Ks + kb * TILE + (st * 32 + l32) * HD;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        Frag kf;
        kf.u = *reinterpret_cast<const uint4*>(kp + (((2 * ks + lhi) ^ kpos_sw) << 3));
        s[st] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf.v, qf[ks].v, s[st], 0, 0, 0);
      }
    }
  };
  // online softmax of tile kt (scores in s, replaced by probabilities), then O^T += V^T P^T from value buffer vb
  auto softmax_pv = [&](floatx16 (&s)[2], int kt, int vb, auto masked) {
    const int kbase = kt * 64;
    if (decltype(masked)::value && kbase + 64 > T) {
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int q = 0; q < 16; ++q) {
          const int key = kbase + st * 32 + 8 * (q >> 2) + 4 * lhi + (q & 3);
          if (key >= T) s[st][q] = -INFINITY;
        }
    }
    float tmax = -INFINITY;
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int q = 0; q < 16; ++q) tmax = fmaxf(tmax, s[st][q]);
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float mnew = fmaxf(mrun, tmax);
    const float moff = mnew * scale_log2e;
    float psum = 0.0f;
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const float p = fast_exp2(fmaf(s[st][q], scale_log2e, -moff));
        s[st][q] = p;
        psum += p;
      }
    if (PIPE && !decltype(masked)::value) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     // one key fragment read
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one MFMA of the next tile's scores
        __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);     // two exponentials of this tile's softmax
        __builtin_amdgcn_sched_group_barrier(0x002, 7, 0);     // seven of its other vector instructions
      }
    }
    if (__any(mnew != mrun)) {
      const float corr = fast_exp2(mrun * scale_log2e - moff);
      lrun *= corr;
#pragma unroll
      for (int i = 0; i < DT; ++i)
#pragma unroll
        for (int q = 0; q < 16; ++q) o[i][q] *= corr;
      mrun = mnew;
    }
    lrun += psum;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int st = t >> 1, j0 = (t & 1) * 8;
      Frag pf;
      pf.u = make_uint4(cvt_pk_bf16(s[st][j0], s[st][j0 + 1]), cvt_pk_bf16(s[st][j0 + 2], s[st][j0 + 3]),
                        cvt_pk_bf16(s[st][j0 + 4], s[st][j0 + 5]), cvt_pk_bf16(s[st][j0 + 6], s[st][j0 + 7]));
      const int ka = 16 * t + vkey0, kb = ka + 8;                  // rows of the two transposing reads
      const int swa = 4 * (ka & 3) + ((ka >> 2) & 3), swb = 4 * (kb & 3) + ((kb >> 2) & 3);
      const uint16_t* va = Vs + vb * TILE + ka * HD + vhalf;
      const uint16_t* vbp = Vs + vb * TILE + kb * HD + vhalf;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const int c = dt * 4 + vchunk0;
        const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)(va + ((c ^ swa) << 3)));
        const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v*)(vbp + ((c ^ swb) << 3)));
        union { short4v h[2]; bf16x8 v; } vf;
        vf.h[0] = lo; vf.h[1] = hi;
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf.v, o[dt], 0, 0, 0);
      }
    }
  };

  const int ntiles = (T + 63) / 64;
  if (!PIPE) {
    issue_k(0, 0);
    issue_v(0, 0);
    for (int kt = 0; kt < ntiles; ++kt) {
      const int buf = kt & 1;
      __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0): this wave's loads of tile kt (nothing else is outstanding)
      __syncthreads();                           // tile kt is in LDS; everyone is done with the other buffer
      if (kt + 1 < ntiles) { issue_k((kt + 1) * 64, buf ^ 1); issue_v((kt + 1) * 64, buf ^ 1); }
      floatx16 s[2];
      scores(s, buf);
      softmax_pv(s, kt, buf, std::true_type());
    }
  } else {
    // The scores of tile kt + 1 are issued before the softmax of tile kt: their MFMAs run while the vector
    // unit takes exponentials.  Keys are therefore fetched two tiles ahead, values one: at the top of
    // iteration kt the wave's outstanding loads are K(kt + 1) and V(kt), both awaited with vmcnt(0);
    // K(kt + 2) then overwrites K(kt) (consumed in iteration kt - 1), V(kt + 1) overwrites V(kt - 1).
    floatx16 sa[2], sb[2];
    issue_k(0, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    if (1 < ntiles) issue_k(64, 1);
    issue_v(0, 0);
    scores(sa, 0);
    // All tiles but the last: no tail mask and no condition between the score MFMAs of tile kt + 1 and the
    // softmax of tile kt, so both sit in one scheduling region; the group barriers ask for one key-fragment
    // read and one MFMA per two exponentials and seven other vector instructions (the wave issues in order:
    // without the interleave the sixteen dependent MFMAs would all be issued before the first exponential).
#define SPECA_ATTN_ITER(kt_, SC, SN)                                                                              \
  {                                                                                                               \
    __builtin_amdgcn_s_waitcnt(0x0F70);                                                                           \
    __syncthreads();                                                                                              \
    if ((kt_) + 2 < ntiles) issue_k(((kt_) + 2) * 64, (kt_) & 1);                                                 \
    issue_v(((kt_) + 1) * 64, ((kt_) + 1) & 1);                                                                   \
    scores(SN, ((kt_) + 1) & 1);                                                                                  \
    softmax_pv(SC, (kt_), (kt_) & 1, std::false_type());                                                          \
  }
    int kt = 0;
    for (; kt + 2 < ntiles; kt += 2) {
      SPECA_ATTN_ITER(kt, sa, sb);
      SPECA_ATTN_ITER(kt + 1, sb, sa);
    }
    if (kt + 1 < ntiles) {                     // two tiles left: kt (scores in sa) and the last one
      SPECA_ATTN_ITER(kt, sa, sb);
      __builtin_amdgcn_s_waitcnt(0x0F70);
      __syncthreads();
      softmax_pv(sb, kt + 1, (kt + 1) & 1, std::true_type());
    } else {                                   // one tile left, its scores are in sa
      __builtin_amdgcn_s_waitcnt(0x0F70);
      __syncthreads();
      softmax_pv(sa, kt, kt & 1, std::true_type());
    }
#undef SPECA_ATTN_ITER
  }

  const float ltot = lrun + __shfl_xor(lrun, 32, 64);
  const float inv = 1.0f / ltot;
  const int q = q0 + wave * 32 + l32;
  if (q < T) {
    uint16_t* op = out + (static_cast<int64_t>(row) * T + q) * ldo + head * HD;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        const int d = dt * 32 + 8 * jj + 4 * lhi;
        uint2 r;
        r.x = cvt_pk_bf16(o[dt][4 * jj] * inv, o[dt][4 * jj + 1] * inv);
        r.y = cvt_pk_bf16(o[dt][4 * jj + 2] * inv, o[dt][4 * jj + 3] * inv);
        *reinterpret_cast<uint2*>(op + d) = r;
      }
  }
}

// Whole-sequence form for T <= 256: one block of 8 waves per (row, head).  Every key and value of the
// head is brought into LDS by one wave of loads issued all at once (a single memory round trip, one
// barrier), each wave then owns 32 queries, holds its complete score row in registers (8 sub-tiles),
// takes the softmax in one pass (no running maximum, no rescaling of O) and runs the second
// contraction over all keys.  At 256 tokens the tiled kernels spend their time in per-tile load
// latency and barriers; this form is bound by one load round trip plus ~90 MFMAs per wave.
constexpr size_t whole_lds_bytes(int HD, bool stage) {
  const int HD16 = (HD + 15) / 16 * 16, HD32 = (HD + 31) / 32 * 32;
  return (static_cast<size_t>(256) * (HD16 + 8) + static_cast<size_t>(HD32) * 256 + (stage ? static_cast<size_t>(8) * 32 * HD : 0)) * sizeof(uint16_t);
}
constexpr bool whole_stages_output(int HD) { return whole_lds_bytes(HD, true) <= 160 * 1024; }

// FULL: T == 256 exactly (the DiT-XL/2 shape): no bounds tests, no ragged sub-tile, so the two contractions and the
// softmax between them are one straight-line region that the scheduler can interleave.
template <int HD, bool FULL>
__global__ __launch_bounds__(512) void attention_mfma_whole_kernel(const uint16_t* __restrict__ qkv, uint16_t* __restrict__ out, int64_t ldo,
                                                                   int T_, int H, float scale_log2e) {
  constexpr int TMAX = 256;
  const int T = FULL ? TMAX : T_;
  constexpr int HD16 = (HD + 15) / 16 * 16, HD32 = (HD + 31) / 32 * 32;
  constexpr int KS = HD16 / 16;         // reduction steps of q k^T
  constexpr int DT = HD32 / 32;         // 32-row tiles of O^T
  constexpr int KST = HD16 + 8;         // LDS row stride of the keys (elements)
  constexpr int CH = HD / 8;            // 16-byte chunks per key/value row
  constexpr int NST = TMAX / 32;        // 32-key sub-tiles
  constexpr int K_CHUNKS = (TMAX * CH + 511) / 512;
  static_assert(HD % 8 == 0, "head_dim must be a multiple of 8");
  static_assert((TMAX / 8) * CH <= 512, "one 8x8 value block per thread");
  extern __shared__ __align__(16) uint16_t smem[];
  uint16_t* Ks = smem;                        // [TMAX][KST]
  uint16_t* Vt = smem + TMAX * KST;           // [HD32][TMAX], see vt_read_off
  uint16_t* Os = Vt + HD32 * TMAX;            // [8 waves][32 queries][HD]: output staging, private to a wave (STAGE_OUT)
  constexpr bool STAGE_OUT = whole_stages_output(HD);

  // blocks b, b + 8, b + 16, ... run on the same XCD: give each XCD a contiguous range of (row, head) pairs, so
  // that a row's q, k and v are pulled into one L2 instead of a slice of every row into all eight
  const int lin = blockIdx.y + gridDim.y * blockIdx.z, total = gridDim.y * gridDim.z;
  const int pair = total % 8 == 0 ? (lin % 8) * (total / 8) + lin / 8 : lin;
  const int row = pair / H, head = pair - row * H;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lhi = lane >> 5;
  const int64_t D = static_cast<int64_t>(H) * HD;
  const uint16_t* base = qkv + static_cast<int64_t>(row) * T * 3 * D + head * HD;

  // all global loads first: keys, one 8x8 value block, the wave's queries
  uint4 rk[K_CHUNKS], rv[8];
#pragma unroll
  for (int c = 0; c < K_CHUNKS; ++c) {
    const int id = tid + c * 512;
    const int key = id / CH, dc = id - key * CH;
    rk[c] = (id < TMAX * CH && key < T) ? *reinterpret_cast<const uint4*>(base + static_cast<int64_t>(key) * 3 * D + D + dc * 8) : make_uint4(0, 0, 0, 0);
  }
  const bool v_thread = tid < (TMAX / 8) * CH;
  const int v_kb = tid / CH, v_dc = tid % CH;   // 8x8 block: keys v_kb*8.., dims v_dc*8..
  if (v_thread) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int key = v_kb * 8 + i;
      rv[i] = key < T ? *reinterpret_cast<const uint4*>(base + static_cast<int64_t>(key) * 3 * D + 2 * D + v_dc * 8) : make_uint4(0, 0, 0, 0);
    }
  }
  Frag qf[KS];
  const int q = wave * 32 + l32;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const int d = ks * 16 + lhi * 8;
    qf[ks].u = (q < T && d < HD) ? *reinterpret_cast<const uint4*>(base + static_cast<int64_t>(q) * 3 * D + d) : make_uint4(0, 0, 0, 0);
  }

  // zero padding: key columns [HD, HD16) and value rows [HD, HD32)
  if (HD16 > HD)
    for (int i = tid; i < TMAX * (HD16 - HD); i += 512) Ks[(i / (HD16 - HD)) * KST + HD + i % (HD16 - HD)] = 0;
  // (with a spare row, row HD of V^T is all ones: row HD of O^T is then the sum of the probabilities as the matrix
  // cores saw them, rounded to bf16 like the numerator)
  constexpr bool ONES = HD32 > HD;
  if (HD32 > HD)
    for (int i = tid; i < (HD32 - HD) * TMAX; i += 512) Vt[HD * TMAX + i] = i < TMAX ? 0x3F80 : 0;
#pragma unroll
  for (int c = 0; c < K_CHUNKS; ++c) {
    const int id = tid + c * 512;
    const int key = id / CH, dc = id - key * CH;
    if (id < TMAX * CH) *reinterpret_cast<uint4*>(Ks + key * KST + dc * 8) = rk[c];
  }
  if (v_thread) {
    // rv[i] = 8 dims of key i  ->  8 rows (dims) of 8 keys
    const uint32_t w[8][4] = {{rv[0].x, rv[0].y, rv[0].z, rv[0].w}, {rv[1].x, rv[1].y, rv[1].z, rv[1].w},
                              {rv[2].x, rv[2].y, rv[2].z, rv[2].w}, {rv[3].x, rv[3].y, rv[3].z, rv[3].w},
                              {rv[4].x, rv[4].y, rv[4].z, rv[4].w}, {rv[5].x, rv[5].y, rv[5].z, rv[5].w},
                              {rv[6].x, rv[6].y, rv[6].z, rv[6].w}, {rv[7].x, rv[7].y, rv[7].z, rv[7].w}};
#pragma unroll
    for (int dd = 0; dd < 8; ++dd) {
      uint32_t r[4];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const uint32_t a = w[2 * kk][dd >> 1], b = w[2 * kk + 1][dd >> 1];
        r[kk] = (dd & 1) ? ((a >> 16) | (b & 0xFFFF0000u)) : ((a & 0xFFFFu) | (b << 16));
      }
      int lo_, hi_;
      vt_write_off<TMAX>(v_dc * 8 + dd, v_kb, &lo_, &hi_);
      *reinterpret_cast<uint2*>(Vt + lo_) = make_uint2(r[0], r[1]);
      *reinterpret_cast<uint2*>(Vt + hi_) = make_uint2(r[2], r[3]);
    }
  }
  __syncthreads();
  if (!FULL && wave * 32 >= T) return;         // no barrier after this point

  const int nst = FULL ? NST : (T + 31) / 32;  // sub-tiles that hold keys
  floatx16 s[NST];
  float tmax = -INFINITY;
#pragma unroll
  for (int st = 0; st < NST; ++st) {
#pragma unroll
    for (int e = 0; e < 16; ++e) s[st][e] = 0.0f;
    if (st < nst) {
      const uint16_t* kp = Ks + (st * 32 + l32) * KST + lhi * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        Frag kf;
        kf.u = *reinterpret_cast<const uint4*>(kp + ks * 16);
        s[st] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf.v, qf[ks].v, s[st], 0, 0, 0);
      }
      if (st * 32 + 32 > T) {                  // ragged last sub-tile
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int key = st * 32 + 8 * (e >> 2) + 4 * lhi + (e & 3);
          if (key >= T) s[st][e] = -INFINITY;
        }
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) tmax = fmaxf(tmax, s[st][e]);
    }
  }
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));     // maximum of the raw scores; scale and log2(e) enter in the fma below
  const float moff = tmax * scale_log2e;
  float psum = 0.0f;
  auto exps = [&](int st) {                      // probabilities of one sub-tile, in place
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const float p = fast_exp2(fmaf(s[st][e], scale_log2e, -moff));
      s[st][e] = p;
      if (!ONES) psum += p;
    }
  };
  floatx16 o[DT];
#pragma unroll
  for (int i = 0; i < DT; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[i][e] = 0.0f;
  // V^T fragment addresses: chunk (2t + h) ^ swz(d) = 16 (t >> 3) + ((2 (t & 7)) ^ (h ^ swz(d))) because swz < 16 and h < 2,
  // so eight per-lane offsets per 32-row tile (one for each t & 7) and an immediate for t >> 3 replace the arithmetic per read
  // (24 registers at head_dim 72; at head_dim 128 the table would spill, so the offsets are formed per read there)
  constexpr bool VTAB = DT <= 3;
  int vto[VTAB ? DT : 1][8];
#pragma unroll
  for (int dt = 0; dt < (VTAB ? DT : 0); ++dt) {
    const int dd = dt * 32 + l32, y = lhi ^ vt_swz<TMAX>(dd);
#pragma unroll
    for (int b = 0; b < 8; ++b) vto[dt][b] = dd * TMAX + (((2 * b) ^ y) << 3);
  }
  // the exponentials of sub-tile st + 1 are issued with the second contraction of sub-tile st
  if (0 < nst) exps(0);
#pragma unroll
  for (int st = 0; st < NST; ++st) {
    if (st < nst) {
      if (st + 1 < NST && st + 1 < nst) exps(st + 1);
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const int t = 2 * st + hh, j0 = hh * 8;   // accumulator entries j0 .. j0+7 of sub-tile st: 16 keys
        Frag pf;
        pf.u = make_uint4(cvt_pk_bf16(s[st][j0], s[st][j0 + 1]), cvt_pk_bf16(s[st][j0 + 2], s[st][j0 + 3]),
                          cvt_pk_bf16(s[st][j0 + 4], s[st][j0 + 5]), cvt_pk_bf16(s[st][j0 + 6], s[st][j0 + 7]));
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          Frag vf;
          vf.u = *reinterpret_cast<const uint4*>(Vt + (VTAB ? vto[VTAB ? dt : 0][t & 7] + (t >> 3) * 128 : vt_read_off<TMAX>(dt * 32 + l32, t, lhi)));
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf.v, o[dt], 0, 0, 0);
        }
      }
    }
  }
  // row HD of O^T sits in accumulator entry (HD % 32 / 8) * 4 of the last tile, in the lanes with lhi == 0
  const float ltot = ONES ? __shfl(o[DT - 1][(HD % 32 / 8) * 4], l32, 64) : psum + __shfl_xor(psum, 32, 64);
  const float inv = 1.0f / ltot;
  // A lane holds one query's output in 8-byte pieces 2304 bytes apart from its neighbour's: the wave re-lays its
  // 32 x HD tile through its own piece of LDS and stores whole 16-byte chunks, a query's HD values contiguous.
  if (!STAGE_OUT) {                            // no LDS to spare: 8-byte stores straight from the accumulators
    if (q < T) {
      uint16_t* op = out + (static_cast<int64_t>(row) * T + q) * ldo + head * HD;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int d = dt * 32 + 8 * jj + 4 * lhi;
          if (d < HD) {
            uint2 r;
            r.x = cvt_pk_bf16(o[dt][4 * jj] * inv, o[dt][4 * jj + 1] * inv);
            r.y = cvt_pk_bf16(o[dt][4 * jj + 2] * inv, o[dt][4 * jj + 3] * inv);
            *reinterpret_cast<uint2*>(op + d) = r;
          }
        }
    }
    return;
  }
  uint16_t* ow = Os + wave * 32 * HD;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const int d = dt * 32 + 8 * jj + 4 * lhi;
      if (d < HD) {
        uint2 r;
        r.x = cvt_pk_bf16(o[dt][4 * jj] * inv, o[dt][4 * jj + 1] * inv);
        r.y = cvt_pk_bf16(o[dt][4 * jj + 2] * inv, o[dt][4 * jj + 3] * inv);
        *reinterpret_cast<uint2*>(ow + l32 * HD + d) = r;
      }
    }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");       // the wave's LDS writes before its reads below
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  uint16_t* ob = out + (static_cast<int64_t>(row) * T + wave * 32) * ldo + head * HD;
#pragma unroll
  for (int c0 = 0; c0 < 32 * CH; c0 += 64) {
    const int c = c0 + lane;
    const int qq = c / CH, dc = c - qq * CH;
    if (c < 32 * CH && wave * 32 + qq < T)
      *reinterpret_cast<uint4*>(ob + static_cast<int64_t>(qq) * ldo + dc * 8) = *reinterpret_cast<const uint4*>(ow + qq * HD + dc * 8);
  }
}

template <int HD>
Error launch_hd(const void* qkv, void* out, int64_t ldo, int rows, int T, int H, hipStream_t st) {
  constexpr int HD16 = (HD + 15) / 16 * 16, HD32 = (HD + 31) / 32 * 32;
  const size_t smem = static_cast<size_t>(2) * (64 * (HD16 + 8) + HD32 * 64) * sizeof(uint16_t);
  // (the whole-sequence kernel stores 16-byte chunks of the output when it stages them through LDS)
  if (T <= 256 && (!whole_stages_output(HD) || (ldo % 8 == 0 && reinterpret_cast<uintptr_t>(out) % 16 == 0))) {
    constexpr size_t smem_w = whole_lds_bytes(HD, whole_stages_output(HD));
    static bool attr_w = false;
    if (smem_w > 64 * 1024 && !attr_w) {
      SPECA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(attention_mfma_whole_kernel<HD, false>), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(smem_w)));
      SPECA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(attention_mfma_whole_kernel<HD, true>), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(smem_w)));
      attr_w = true;
    }
    const float sl2 = 1.4426950408889634f / sqrtf(static_cast<float>(HD));
    if (T == 256) attention_mfma_whole_kernel<HD, true><<<dim3(1, H, rows), 512, smem_w, st>>>(static_cast<const uint16_t*>(qkv), static_cast<uint16_t*>(out), ldo, T, H, sl2);
    else attention_mfma_whole_kernel<HD, false><<<dim3(1, H, rows), 512, smem_w, st>>>(static_cast<const uint16_t*>(qkv), static_cast<uint16_t*>(out), ldo, T, H, sl2);
    SPECA_HIP(hipGetLastError());
    return ok();
  }
  // head_dim 128: direct-to-LDS tiles with the transposing read, scores of the next tile under the softmax
  if (HD == 128) {
    constexpr size_t smem_d = static_cast<size_t>(4) * 64 * 128 * sizeof(uint16_t);
    dim3 grid_d((T + 127) / 128, H, rows);
    const float sl2 = 1.4426950408889634f / sqrtf(128.0f);
    attention_dma_kernel<true><<<grid_d, 256, smem_d, st>>>(static_cast<const uint16_t*>(qkv), static_cast<uint16_t*>(out), ldo, T, H, sl2);
    SPECA_HIP(hipGetLastError());
    return ok();
  }
  auto kern = attention_mfma_kernel<HD>;
  static bool attr_set = false;
  if (smem > 64 * 1024 && !attr_set) {
    SPECA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(attention_mfma_kernel<HD>), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(smem)));
    attr_set = true;
  }
  dim3 grid((T + 127) / 128, H, rows);
  const float scale_log2e = 1.4426950408889634f / sqrtf(static_cast<float>(HD));
  kern<<<grid, 256, smem, st>>>(static_cast<const uint16_t*>(qkv), static_cast<uint16_t*>(out), ldo, T, H, scale_log2e);
  SPECA_HIP(hipGetLastError());
  return ok();
}

}  // namespace

bool attention_mfma_supported(const void* qkv, const void* out, int64_t ldo, int H, int hd) {
  return (hd == 64 || hd == 72 || hd == 128) && ldo % 4 == 0 && reinterpret_cast<uintptr_t>(qkv) % 16 == 0 && reinterpret_cast<uintptr_t>(out) % 8 == 0;
}

Error launch_attention_mfma(const void* qkv, void* out, int64_t ldo, int rows, int T, int H, int hd, hipStream_t st) {
  if (rows > 65535 || H > 65535) SPECA_FAIL(SPECA_EINVAL, "attention: grid too large");
  switch (hd) {
    case 64: return launch_hd<64>(qkv, out, ldo, rows, T, H, st);
    case 72: return launch_hd<72>(qkv, out, ldo, rows, T, H, st);
    case 128: return launch_hd<128>(qkv, out, ldo, rows, T, H, st);
  }
  SPECA_FAIL(SPECA_EUNSUPPORTED, "attention: head_dim %d has no MFMA kernel", hd);
}

}  // namespace speca
