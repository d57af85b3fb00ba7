// What joins the probe linears of a decoder block during a candidate's scoring pass
// (Sec. 2.2: a query is a teacher-forced scoring pass under the candidate's weights;
// Sec. 3.1: packed variable-length sequences): residual sum + normalisation, and causal
// self-attention over each packed sequence.  None of it has perturbed parameters, so it is
// the same for every candidate and takes no candidate table.
//
//   k_add_norm_bf16 / k_add_norm_any   h = x + res, y = LayerNorm(h) or RMSNorm(h); one wave per row,
//                                      the row stays in registers between the passes (HBM-bound)
//   k_attention_bf16                   online-softmax attention on 16x16x32 bf16 MFMA, head_dim 128
//   k_attention_f32                    plain fp32 attention on the vector ALU (any head_dim <= 256)
//   k_qk_norm_rope_*                   per-head RMS norm of queries and keys + rotary embedding, in place
//                                      (the Qwen3 family; its gated MLP is an epilogue of the probe linear)
#include "zo_device.hpp"
#include "zo_internal.hpp"

namespace zo {
namespace {

typedef __attribute__((address_space(3))) void lds_void;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ void block_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// ------------------------------------------------------------------ add + norm

constexpr int kNormWaves = 4;   // waves per workgroup, one row each at a time

// bf16 rows with d % 8 == 0 and d <= kChunks * 512: lane l owns the 8 elements starting at
// (c*64 + l)*8 of chunk c.  Exact two-pass moments in fp32 on the register copy of the row.
// A workgroup covers rows_per_wave * 4 consecutive rows; gamma and beta are staged once per
// workgroup in LDS (re-reading them per row from L2 would move four times the bytes of the
// row itself), in the order the lanes read them: the two 16-byte halves of a lane's 8 values
// sit in separate planes so that consecutive lanes read consecutive 16-byte words.
template <int kChunks>
__global__ __launch_bounds__(kNormWaves* kWave) void k_add_norm_bf16(NormArgs a, int rows_per_wave) {
  __shared__ __attribute__((aligned(16))) float s_gamma[kChunks * 512];
  __shared__ __attribute__((aligned(16))) float s_beta[kChunks * 512];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (a.Y) {
    for (int e = threadIdx.x * 4; e < a.d; e += kNormWaves * kWave * 4) {
      const int at = (e >> 9) * 512 + ((e >> 2) & 1) * 256 + ((e & 511) >> 3) * 4;
      *reinterpret_cast<float4*>(&s_gamma[at]) = *reinterpret_cast<const float4*>(a.gamma + e);
      *reinterpret_cast<float4*>(&s_beta[at]) =
          a.beta ? *reinterpret_cast<const float4*>(a.beta + e) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    __syncthreads();
  }
  const float inv_d = 1.0f / (float)a.d;
  for (int it = 0; it < rows_per_wave; ++it) {
    const int row = (blockIdx.x * rows_per_wave + it) * kNormWaves + wave;
    if (row >= a.T) return;
    const bf16_t* x = (const bf16_t*)a.X + (int64_t)row * a.ldx;
    const bf16_t* res = a.R ? (const bf16_t*)a.R + (int64_t)row * a.ldr : nullptr;
    bf16_t* hs = a.Hsum ? (bf16_t*)a.Hsum + (int64_t)row * a.ldh : nullptr;
    float v[kChunks][8];
    float sum = 0.f, sumsq = 0.f;
#pragma unroll
    for (int c = 0; c < kChunks; ++c) {
      const int e0 = (c * kWave + lane) * 8;
      if (e0 < a.d) {
        const u32x4 xv = *reinterpret_cast<const u32x4*>(x + e0);
        u32x4 rv = {0u, 0u, 0u, 0u};
        if (res) rv = *reinterpret_cast<const u32x4*>(res + e0);
        u32x4 hv;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float lo = __uint_as_float(xv[i] << 16), hi = __uint_as_float(xv[i] & 0xFFFF0000u);
          if (res) {
            // the sum is stored as bf16, and it is that stored value which is normalised
            const uint32_t p =
                pack_bf16x2(lo + __uint_as_float(rv[i] << 16), hi + __uint_as_float(rv[i] & 0xFFFF0000u));
            hv[i] = p;
            lo = __uint_as_float(p << 16);
            hi = __uint_as_float(p & 0xFFFF0000u);
          }
          v[c][2 * i] = lo;
          v[c][2 * i + 1] = hi;
          sum += lo + hi;
          sumsq += lo * lo + hi * hi;
        }
        if (res && hs) *reinterpret_cast<u32x4*>(hs + e0) = hv;
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[c][i] = 0.f;
      }
    }
    if (!a.Y) continue;
    float mean = 0.f, rstd;
    if (a.kind == 0) {
      mean = wave_sum(sum) * inv_d;
      float dev = 0.f;
#pragma unroll
      for (int c = 0; c < kChunks; ++c)
        if ((c * kWave + lane) * 8 < a.d) {
#pragma unroll
          for (int i = 0; i < 8; ++i) dev += (v[c][i] - mean) * (v[c][i] - mean);
        }
      rstd = 1.0f / sqrtf(wave_sum(dev) * inv_d + a.eps);
    } else {
      rstd = 1.0f / sqrtf(wave_sum(sumsq) * inv_d + a.eps);
    }
    bf16_t* y = (bf16_t*)a.Y + (int64_t)row * a.ldy;
#pragma unroll
    for (int c = 0; c < kChunks; ++c) {
      const int e0 = (c * kWave + lane) * 8;
      if (e0 < a.d) {
        const float4 g0 = *reinterpret_cast<const float4*>(&s_gamma[c * 512 + lane * 4]);
        const float4 g1 = *reinterpret_cast<const float4*>(&s_gamma[c * 512 + 256 + lane * 4]);
        const float4 b0 = *reinterpret_cast<const float4*>(&s_beta[c * 512 + lane * 4]);
        const float4 b1 = *reinterpret_cast<const float4*>(&s_beta[c * 512 + 256 + lane * 4]);
        u32x4 o;
        o[0] = pack_bf16x2((v[c][0] - mean) * rstd * g0.x + b0.x, (v[c][1] - mean) * rstd * g0.y + b0.y);
        o[1] = pack_bf16x2((v[c][2] - mean) * rstd * g0.z + b0.z, (v[c][3] - mean) * rstd * g0.w + b0.w);
        o[2] = pack_bf16x2((v[c][4] - mean) * rstd * g1.x + b1.x, (v[c][5] - mean) * rstd * g1.y + b1.y);
        o[3] = pack_bf16x2((v[c][6] - mean) * rstd * g1.z + b1.z, (v[c][7] - mean) * rstd * g1.w + b1.w);
        *reinterpret_cast<u32x4*>(y + e0) = o;
      }
    }
  }
}

__device__ __forceinline__ float ld_elem(const float* p, int64_t i) { return p[i]; }
__device__ __forceinline__ float ld_elem(const bf16_t* p, int64_t i) { return bf16_to_f32(p[i]); }
__device__ __forceinline__ float st_round(float*, float v) { return v; }
__device__ __forceinline__ float st_round(bf16_t*, float v) { return bf16_round(v); }
__device__ __forceinline__ void st_elem(float* p, int64_t i, float v) { p[i] = v; }
__device__ __forceinline__ void st_elem(bf16_t* p, int64_t i, float v) { p[i] = f32_to_bf16(v); }

// Any width and either storage type: one wave per row, the row is re-read from memory per pass.
// A lane reads back only elements it wrote itself, so Hsum may alias X.
template <typename Tio>
__global__ __launch_bounds__(kNormWaves* kWave) void k_add_norm_any(NormArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = blockIdx.x * kNormWaves + wave;
  if (row >= a.T) return;
  const Tio* x = (const Tio*)a.X + (int64_t)row * a.ldx;
  const Tio* res = a.R ? (const Tio*)a.R + (int64_t)row * a.ldr : nullptr;
  Tio* hs = a.Hsum ? (Tio*)a.Hsum + (int64_t)row * a.ldh : nullptr;
  const bool stored = res && hs;
  float sum = 0.f, sumsq = 0.f;
  for (int e = lane; e < a.d; e += kWave) {
    float h = ld_elem(x, e);
    if (res) h = st_round((Tio*)nullptr, h + ld_elem(res, e));
    if (stored) st_elem(hs, e, h);
    sum += h;
    sumsq += h * h;
  }
  if (!a.Y) return;
  auto value = [&](int e) {
    if (stored) return ld_elem((const Tio*)hs, e);
    float h = ld_elem(x, e);
    if (res) h = st_round((Tio*)nullptr, h + ld_elem(res, e));
    return h;
  };
  const float inv_d = 1.0f / (float)a.d;
  float mean = 0.f, rstd;
  if (a.kind == 0) {
    mean = wave_sum(sum) * inv_d;
    float dev = 0.f;
    for (int e = lane; e < a.d; e += kWave) {
      const float t = value(e) - mean;
      dev += t * t;
    }
    rstd = 1.0f / sqrtf(wave_sum(dev) * inv_d + a.eps);
  } else {
    rstd = 1.0f / sqrtf(wave_sum(sumsq) * inv_d + a.eps);
  }
  Tio* y = (Tio*)a.Y + (int64_t)row * a.ldy;
  for (int e = lane; e < a.d; e += kWave)
    st_elem(y, e, (value(e) - mean) * rstd * a.gamma[e] + (a.beta ? a.beta[e] : 0.f));
}

// ------------------------------------------------------------------ attention, fp32

// Largest i with cu[i] <= t (cu[0] = 0 <= t < cu[S]): the sequence that holds row t.
__device__ __forceinline__ int seq_of_row(const int32_t* cu, int S, int t) {
  int lo = 0, hi = S;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (cu[mid] <= t) lo = mid; else hi = mid - 1;
  }
  return lo;
}

constexpr int kAttnF32MaxDh = 256;

// One wave per (row, head): scores in two passes (maximum, then weights), values accumulated
// with lanes over the head dimension.
__global__ __launch_bounds__(kWave) void k_attention_f32(AttnArgs a) {
  __shared__ float s_q[kAttnF32MaxDh];
  __shared__ float s_p[kWave];
  const int lane = threadIdx.x;
  const int t = blockIdx.x, h = blockIdx.y, g = h / a.group;
  const int dh = a.dh;
  const int a0 = a.cu[seq_of_row(a.cu, a.S, t)];
  const int nkeys = t - a0 + 1;
  const float* q = (const float*)a.Q + (int64_t)t * a.ldq + h * dh;
  const float* Kb = (const float*)a.K + (int64_t)a0 * a.ldk + g * dh;
  const float* Vb = (const float*)a.V + (int64_t)a0 * a.ldv + g * dh;
  for (int d = lane; d < dh; d += kWave) s_q[d] = q[d];
  __syncthreads();
  auto score = [&](int j) {
    const float* k = Kb + (int64_t)j * a.ldk;
    float s = 0.f;
    for (int d = 0; d < dh; ++d) s += s_q[d] * k[d];
    return s * a.scale;
  };
  float mx = -INFINITY;
  for (int j = lane; j < nkeys; j += kWave) mx = fmaxf(mx, score(j));
  mx = wave_max(mx);
  float acc[kAttnF32MaxDh / kWave] = {0.f, 0.f, 0.f, 0.f};
  float lsum = 0.f;
  for (int base = 0; base < nkeys; base += kWave) {
    const int j = base + lane;
    const float p = j < nkeys ? expf(score(j) - mx) : 0.f;
    lsum += p;
    s_p[lane] = p;
    __syncthreads();
    const int cnt = min(kWave, nkeys - base);
    for (int jj = 0; jj < cnt; ++jj) {
      const float pj = s_p[jj];
      const float* v = Vb + (int64_t)(base + jj) * a.ldv;
#pragma unroll
      for (int c = 0; c < kAttnF32MaxDh / kWave; ++c)
        if (lane + c * kWave < dh) acc[c] += pj * v[lane + c * kWave];
    }
    __syncthreads();
  }
  const float inv = 1.0f / wave_sum(lsum);
  float* o = (float*)a.O + (int64_t)t * a.ldo + h * dh;
#pragma unroll
  for (int c = 0; c < kAttnF32MaxDh / kWave; ++c)
    if (lane + c * kWave < dh) o[lane + c * kWave] = acc[c] * inv;
}

// ------------------------------------------------------------------ attention, bf16 MFMA

constexpr int kBQ = 128;            // query rows per workgroup (32 per wave)
constexpr int kBKV = 64;            // keys per step
constexpr int kDh = 128;            // head dimension of this kernel
constexpr int kAttnWaves = 4;
constexpr int kKStage = kBKV * kDh * 2;   // 16 KiB: keys x head dim, 256-byte rows
constexpr int kVStage = kDh * kBKV * 2;   // 16 KiB: head dim x keys (transposed), 128-byte rows

// Swizzle key of an LDS row: the 16-byte chunk c of row `row` is stored at chunk c ^ key.  The 16
// rows a fragment read touches are {8*(i/4) + i%4 : i < 16} (+ a multiple of 4 and of 32), over
// which the key takes each of its 8 values exactly twice: every read is bank-conflict free.
__device__ __forceinline__ int swz_key(int row) { return ((row >> 1) & 1) | (((row >> 3) & 3) << 1); }

// Finds the (sequence, query block) pair behind slot w: sequences are walked 64 at a time and a
// wave-wide prefix sum of their block counts locates the slot.  Every wave of the workgroup
// computes the same answer.  Returns false when w is past the last pair.
__device__ __forceinline__ bool find_query_block(const int32_t* cu, int S, int w, int lane, int& seq, int& qb) {
  int base = 0;
  for (int s0 = 0; s0 < S; s0 += kWave) {
    const int i = s0 + lane;
    const int nb = i < S ? (cu[i + 1] - cu[i] + kBQ - 1) / kBQ : 0;
    int inc = nb;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const int up = __shfl_up(inc, o);
      if (lane >= o) inc += up;
    }
    const int excl = base + inc - nb;
    const unsigned long long hit = __ballot(w >= excl && w < excl + nb);
    if (hit) {
      const int src = __ffsll((long long)hit) - 1;
      seq = s0 + src;
      qb = w - __shfl(excl, src);
      return true;
    }
    base += __shfl(inc, kWave - 1);
  }
  return false;
}

// Causal attention of one (sequence, head, block of 128 query rows).
//
// Both products are computed transposed so that every per-query quantity lives in the lane that
// owns that query's column: S^T = K Q^T (A = keys from LDS, B = queries held in registers) and
// O^T = V^T P^T (A = transposed values from LDS, B = the weights just computed).  In the 16x16
// result layout lane l holds column l%16 (a query) and rows 4*(l/16)+v; the 16 A-rows of a
// tile are chosen as {8*(i/4) + i%4} (+4 for the second tile of a pair), so that over a pair
// of tiles a lane holds 8 consecutive keys (resp. head-dim elements): exactly the k-group it must
// supply as B operand of the second product (resp. one 16-byte store of the output row).  The
// running maximum, the rescaling factor and the normaliser are then per-lane scalars and P never
// leaves registers.
//
// Keys are fetched global->LDS directly (the swizzle is applied on the source address); values
// pass through registers because they are transposed on the way (4 keys x 8 head-dim elements
// per thread, written as 8-byte key groups).  Both are double-buffered: the loads of step j+1
// are issued before the products of step j.  Rows past the end of the sequence are clamped to
// its last row and are always masked by the causal test.
__global__ __launch_bounds__(kAttnWaves* kWave, 2) void k_attention_bf16(AttnArgs a) {
  __shared__ __attribute__((aligned(1024))) char s_k[2][kKStage];
  __shared__ __attribute__((aligned(1024))) char s_v[2][kVStage];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r16 = lane & 15, g = lane >> 4;
  int seq, qb;
  // One-dimensional grid, heads fastest: the slots past the last query block (the grid is an upper bound) are
  // the last workgroups dispatched instead of a burst after every head, and the query heads that share a
  // key/value head run next to each other (ragged Qwen3-shaped batch: 187 -> 166 us).
  const int slot_id = blockIdx.x / a.n_heads;
  if (!find_query_block(a.cu, a.S, slot_id, lane, seq, qb)) return;
  const int h = blockIdx.x - slot_id * a.n_heads, kvh = h / a.group;
  const int row_a = a.cu[seq], row_b = a.cu[seq + 1];       // the sequence is rows [row_a, row_b)
  const int q0 = row_a + qb * kBQ;
  const int q_last = min(q0 + kBQ, row_b) - 1;
  const int n_steps = (q_last - row_a) / kBKV + 1;
  const int wq0 = q0 + wave * 32;                            // this wave's first query row
  const bool wave_valid = wq0 < row_b;
  const int wq_last = min(wq0 + 31, row_b - 1);

  const bf16_t* Kh = (const bf16_t*)a.K + kvh * kDh;
  const bf16_t* Vh = (const bf16_t*)a.V + kvh * kDh;

  // ---- queries: B fragments, lane (r16, g) holds Q[row r16 of tile qt][32 ks + 8 g .. + 8]
  bf16x8 qf[2][4];
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    const int qrow = min(wq0 + qt * 16 + r16, row_b - 1);
    const bf16_t* qp = (const bf16_t*)a.Q + (int64_t)qrow * a.ldq + h * kDh + g * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) qf[qt][ks] = load_frag(qp + ks * 32);
  }

  // ---- per-lane addressing of the loads
  // keys: load i of a wave fills the 1 KiB block wave*4 + i of the stage = 4 rows of 256 B
  int k_row[4], k_lch[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    k_row[i] = (wave * 4 + i) * 4 + (lane >> 4);
    k_lch[i] = (lane & 15) ^ swz_key(k_row[i]);
  }
  // values: 4 keys (4 kg .. 4 kg + 3) x 8 head-dim elements (8 dhg ..) per thread
  const int dhg = lane & 15, kg = wave * 4 + (lane >> 4);
  const int frag_key = swz_key(8 * (r16 >> 2) + (r16 & 3));   // swizzle key of this lane's fragment rows
  const int frag_row = 8 * (r16 >> 2) + (r16 & 3);

  auto issue_keys = [&](int step, int stage) {
    const int j0 = row_a + step * kBKV;
    const int last_rel = row_b - 1 - j0;
    const bf16_t* base = Kh + (int64_t)j0 * a.ldk;
    const int64_t bytes = ((int64_t)min(last_rel, kBKV - 1) * a.ldk + kDh) * 2;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)bytes, 0x00020000);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t off = (uint32_t)min(k_row[i], last_rel) * (uint32_t)(a.ldk * 2) + k_lch[i] * 16;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)(&s_k[stage][0] + (wave * 4 + i) * 1024), 16, (int)off,
                                               0, 0, 0);
    }
  };
  auto load_values = [&](int step, u32x4 (&vr)[4]) {
    const int j0 = row_a + step * kBKV;
    const int last_rel = row_b - 1 - j0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int key = min(kg * 4 + i, last_rel);
      vr[i] = *reinterpret_cast<const u32x4*>(Vh + (int64_t)(j0 + key) * a.ldv + dhg * 8);
    }
  };
  auto store_values = [&](int stage, const u32x4 (&vr)[4]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int d = dhg * 8 + e;
      const int w = e >> 1;
      uint32_t lo, hi;   // keys (0,1) and (2,3) of head-dim element d
      if (e & 1) {
        lo = (vr[0][w] >> 16) | (vr[1][w] & 0xFFFF0000u);
        hi = (vr[2][w] >> 16) | (vr[3][w] & 0xFFFF0000u);
      } else {
        lo = (vr[0][w] & 0xFFFFu) | (vr[1][w] << 16);
        hi = (vr[2][w] & 0xFFFFu) | (vr[3][w] << 16);
      }
      const int off = d * 128 + ((((kg >> 1) ^ swz_key(d)) << 4) | ((kg & 1) << 3));
      *reinterpret_cast<uint2*>(&s_v[stage][off]) = make_uint2(lo, hi);
    }
  };

  f32x4 oacc[4][2][2];   // [dh pair][half][query tile]
#pragma unroll
  for (int dp = 0; dp < 4; ++dp)
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int qt = 0; qt < 2; ++qt) oacc[dp][hf][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};
  const float sl2 = a.scale * 1.4426950408889634f;   // scores are kept in base-2 units

  u32x4 vr[4];
  issue_keys(0, 0);
  load_values(0, vr);
  store_values(0, vr);
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  block_barrier();

  for (int step = 0; step < n_steps; ++step) {
    const int cur = step & 1;
    const bool more = step + 1 < n_steps;
    if (more) {
      issue_keys(step + 1, cur ^ 1);
      load_values(step + 1, vr);
    }
    const int j0 = row_a + step * kBKV;
    if (wave_valid && j0 <= wq_last) {
      // ---- S^T = K Q^T for 4 key tiles x 2 query tiles
      f32x4 sacc[2][2][2];   // [key pair][half][query tile]
#pragma unroll
      for (int tp = 0; tp < 2; ++tp)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          const char* krow = &s_k[cur][0] + (32 * tp + 4 * hf + frag_row) * 256;
          bf16x8 kf[4];
#pragma unroll
          for (int ks = 0; ks < 4; ++ks)
            kf[ks] = *reinterpret_cast<const bf16x8*>(krow + (((ks * 4 + g) ^ frag_key) << 4));
#pragma unroll
          for (int qt = 0; qt < 2; ++qt) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[ks], qf[qt][ks], acc, 0, 0, 0);
            sacc[tp][hf][qt] = acc;
          }
        }
      // ---- online softmax; lane (g, r16) holds, for query r16 of tile qt, keys 32 tp + 8 g + 4 hf + v
      const bool diagonal = j0 + kBKV - 1 > wq0;
      bf16x8 pf[2][2];   // [query tile][k-step = key pair]
#pragma unroll
      for (int qt = 0; qt < 2; ++qt) {
        const int qrow = min(wq0 + qt * 16 + r16, row_b - 1);
        float mx = m_run[qt];
#pragma unroll
        for (int tp = 0; tp < 2; ++tp)
#pragma unroll
          for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              float s = sacc[tp][hf][qt][v] * sl2;
              if (diagonal && j0 + 32 * tp + 8 * g + 4 * hf + v > qrow) s = -INFINITY;
              sacc[tp][hf][qt][v] = s;
              mx = fmaxf(mx, s);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float alpha = __builtin_amdgcn_exp2f(m_run[qt] - mx);
        m_run[qt] = mx;
        float psum = 0.f;
#pragma unroll
        for (int tp = 0; tp < 2; ++tp) {
          float p[8];
#pragma unroll
          for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              p[hf * 4 + v] = __builtin_amdgcn_exp2f(sacc[tp][hf][qt][v] - mx);
              psum += p[hf * 4 + v];
            }
          u32x4 packed = {pack_bf16x2(p[0], p[1]), pack_bf16x2(p[2], p[3]), pack_bf16x2(p[4], p[5]),
                          pack_bf16x2(p[6], p[7])};
          pf[qt][tp] = __builtin_bit_cast(bf16x8, packed);
        }
        l_run[qt] = l_run[qt] * alpha + psum;
#pragma unroll
        for (int dp = 0; dp < 4; ++dp)
#pragma unroll
          for (int hf = 0; hf < 2; ++hf) oacc[dp][hf][qt] *= alpha;
      }
      // ---- O^T += V^T P^T
#pragma unroll
      for (int dp = 0; dp < 4; ++dp)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
          const char* vrow = &s_v[cur][0] + (32 * dp + 4 * hf + frag_row) * 128;
#pragma unroll
          for (int ks = 0; ks < 2; ++ks) {
            const bf16x8 vf = *reinterpret_cast<const bf16x8*>(vrow + (((ks * 4 + g) ^ frag_key) << 4));
#pragma unroll
            for (int qt = 0; qt < 2; ++qt)
              oacc[dp][hf][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[qt][ks], oacc[dp][hf][qt], 0, 0, 0);
          }
        }
    }
    if (more) store_values(cur ^ 1, vr);
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    block_barrier();
  }

  if (!wave_valid) return;
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    float l = l_run[qt];
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    const float inv = 1.0f / l;
    const int qrow = wq0 + qt * 16 + r16;
    if (qrow < row_b) {
      bf16_t* o = (bf16_t*)a.O + (int64_t)qrow * a.ldo + h * kDh + g * 8;
#pragma unroll
      for (int dp = 0; dp < 4; ++dp) {
        const f32x4 lo = oacc[dp][0][qt], hi = oacc[dp][1][qt];
        u32x4 packed = {pack_bf16x2(lo[0] * inv, lo[1] * inv), pack_bf16x2(lo[2] * inv, lo[3] * inv),
                        pack_bf16x2(hi[0] * inv, hi[1] * inv), pack_bf16x2(hi[2] * inv, hi[3] * inv)};
        *reinterpret_cast<u32x4*>(o + dp * 32) = packed;
      }
    }
  }
}

// ------------------------------------------------------------------ per-head q/k norm + rotary embedding

// Rotation angle of pair i (of dh/2) at position pos: pos * theta^(-2i/dh).
__device__ __forceinline__ float rope_angle(float log2_theta, int i, int dh, int pos) {
  return (float)pos * exp2f(-(float)(2 * i) / (float)dh * log2_theta);
}

// bf16, head dimension 128, in place.  One wave per token, four heads at a time: the 16 lanes of a head
// hold elements 4j..4j+3 and their rotation partners 64+4j..64+4j+3 (j = lane % 16), so the per-head sum
// of squares is four shuffles and the rotation is lane-local.  The token's position and the four
// (cos, sin) pairs of a lane depend on neither the head nor on queries versus keys: they are computed
// once per token, under the first loads.  Heads 0..H-1 are queries, H..H+Hkv-1 keys.
__global__ __launch_bounds__(256) void k_qk_norm_rope_bf16(QkRopeArgs a) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= a.T) return;
  const int heads = a.n_heads + a.n_kv_heads;
  const int groups = (heads + 3) >> 2;
  const int j = lane & 15, hh = lane >> 4;
  auto row_of = [&](int head) -> bf16_t* {
    return head < a.n_heads ? (bf16_t*)a.Q + (int64_t)t * a.ldq + head * 128
                            : (bf16_t*)a.K + (int64_t)t * a.ldk + (head - a.n_heads) * 128;
  };
  auto load = [&](int grp, uint2& lo, uint2& hi) {
    const int head = grp * 4 + hh;
    lo = hi = make_uint2(0u, 0u);
    if (head < heads) {
      const bf16_t* row = row_of(head);
      lo = *reinterpret_cast<const uint2*>(row + 4 * j);
      hi = *reinterpret_cast<const uint2*>(row + 64 + 4 * j);
    }
  };
  uint2 lo, hi;
  load(0, lo, hi);
  float cs[4] = {1.f, 1.f, 1.f, 1.f}, sn[4] = {0.f, 0.f, 0.f, 0.f};
  if (a.theta > 0.f) {
    const int pos = t - a.cu[seq_of_row(a.cu, a.S, t)];
    const float l2t = log2f(a.theta);
#pragma unroll
    for (int e = 0; e < 4; ++e) sincosf(rope_angle(l2t, 4 * j + e, 128, pos), &sn[e], &cs[e]);
  }
  float4 gq0 = make_float4(1.f, 1.f, 1.f, 1.f), gq1 = gq0, gk0 = gq0, gk1 = gq0;
  if (a.gamma_q) {
    gq0 = *reinterpret_cast<const float4*>(a.gamma_q + 4 * j);
    gq1 = *reinterpret_cast<const float4*>(a.gamma_q + 64 + 4 * j);
    gk0 = *reinterpret_cast<const float4*>(a.gamma_k + 4 * j);
    gk1 = *reinterpret_cast<const float4*>(a.gamma_k + 64 + 4 * j);
  }
  for (int grp = 0; grp < groups; ++grp) {
    uint2 nlo, nhi;
    if (grp + 1 < groups) load(grp + 1, nlo, nhi);   // the next four heads travel under this group's arithmetic
    const int head = grp * 4 + hh;
    const bool is_q = head < a.n_heads;
    float x[8];   // [0..3] first half, [4..7] partners
    x[0] = __uint_as_float(lo.x << 16); x[1] = __uint_as_float(lo.x & 0xFFFF0000u);
    x[2] = __uint_as_float(lo.y << 16); x[3] = __uint_as_float(lo.y & 0xFFFF0000u);
    x[4] = __uint_as_float(hi.x << 16); x[5] = __uint_as_float(hi.x & 0xFFFF0000u);
    x[6] = __uint_as_float(hi.y << 16); x[7] = __uint_as_float(hi.y & 0xFFFF0000u);
    if (a.gamma_q) {
      float ss = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) ss += x[e] * x[e];
#pragma unroll
      for (int o = 8; o >= 1; o >>= 1) ss += __shfl_xor(ss, o);
      const float rstd = 1.0f / sqrtf(ss * (1.0f / 128.0f) + a.eps);
      const float4 g0 = is_q ? gq0 : gk0, g1 = is_q ? gq1 : gk1;
      x[0] *= rstd * g0.x; x[1] *= rstd * g0.y; x[2] *= rstd * g0.z; x[3] *= rstd * g0.w;
      x[4] *= rstd * g1.x; x[5] *= rstd * g1.y; x[6] *= rstd * g1.z; x[7] *= rstd * g1.w;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float p = x[e], q = x[4 + e];
      x[e] = p * cs[e] - q * sn[e];
      x[4 + e] = q * cs[e] + p * sn[e];
    }
    if (head < heads) {
      bf16_t* row = row_of(head);
      *reinterpret_cast<uint2*>(row + 4 * j) = make_uint2(pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]));
      *reinterpret_cast<uint2*>(row + 64 + 4 * j) = make_uint2(pack_bf16x2(x[4], x[5]), pack_bf16x2(x[6], x[7]));
    }
    lo = nlo;
    hi = nhi;
  }
}

// Any even head dimension up to 256 and either storage type: one wave per (token, head), lane l holds the
// pairs l and l + 64.  With fp32 storage the angle is formed in double precision, so that positions in the
// thousands still give angles good to fp32 rounding.
template <typename Tio>
__global__ __launch_bounds__(256) void k_qk_norm_rope_any(QkRopeArgs a) {
  const int lane = threadIdx.x & 63;
  const int heads = a.n_heads + a.n_kv_heads;
  const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= (int64_t)a.T * heads) return;
  const int t = (int)(item / heads), head = (int)(item % heads);
  const bool is_q = head < a.n_heads;
  const int dh = a.dh, half = dh >> 1;
  Tio* row = is_q ? (Tio*)a.Q + (int64_t)t * a.ldq + head * dh : (Tio*)a.K + (int64_t)t * a.ldk + (head - a.n_heads) * dh;
  float lo[2], hi[2];
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    const int i = lane + c * kWave;
    lo[c] = i < half ? ld_elem(row, i) : 0.f;
    hi[c] = i < half ? ld_elem(row, half + i) : 0.f;
  }
  if (a.gamma_q) {
    const float ss = wave_sum(lo[0] * lo[0] + hi[0] * hi[0] + lo[1] * lo[1] + hi[1] * hi[1]);
    const float rstd = 1.0f / sqrtf(ss / (float)dh + a.eps);
    const float* gam = is_q ? a.gamma_q : a.gamma_k;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const int i = lane + c * kWave;
      if (i < half) { lo[c] *= rstd * gam[i]; hi[c] *= rstd * gam[half + i]; }
    }
  }
  if (a.theta > 0.f) {
    const int pos = t - a.cu[seq_of_row(a.cu, a.S, t)];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const int i = lane + c * kWave;
      if (i >= half) continue;
      float sn, cs;
      if (sizeof(Tio) == 4) {
        double dsn, dcs;
        sincos((double)pos * exp2(-(double)(2 * i) / (double)dh * log2((double)a.theta)), &dsn, &dcs);
        sn = (float)dsn; cs = (float)dcs;
      } else {
        sincosf(rope_angle(log2f(a.theta), i, dh, pos), &sn, &cs);
      }
      const float p = lo[c], q = hi[c];
      lo[c] = p * cs - q * sn;
      hi[c] = q * cs + p * sn;
    }
  }
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    const int i = lane + c * kWave;
    if (i < half) { st_elem(row, i, lo[c]); st_elem(row, half + i, hi[c]); }
  }
}

}  // namespace

hipError_t launch_qk_norm_rope(const QkRopeArgs& a, hipStream_t st) {
  if (a.T == 0 || (!a.gamma_q && !(a.theta > 0.f))) return hipSuccess;
  const int heads = a.n_heads + a.n_kv_heads;
  auto aligned = [](const void* p, int64_t ld) { return ((uintptr_t)p & 7u) == 0 && ld % 4 == 0; };
  const bool fast = a.bf16 && a.dh == 128 && aligned(a.Q, a.ldq) && aligned(a.K, a.ldk) &&
                    (((uintptr_t)a.gamma_q | (uintptr_t)a.gamma_k) & 15u) == 0;
  if (fast) {
    k_qk_norm_rope_bf16<<<dim3((unsigned)((a.T + 3) / 4)), 256, 0, st>>>(a);
  } else {
    const int64_t items = (int64_t)a.T * heads;
    if (a.bf16) k_qk_norm_rope_any<bf16_t><<<dim3((unsigned)((items + 3) / 4)), 256, 0, st>>>(a);
    else k_qk_norm_rope_any<float><<<dim3((unsigned)((items + 3) / 4)), 256, 0, st>>>(a);
  }
  return hipGetLastError();
}

hipError_t launch_add_norm(const NormArgs& a, hipStream_t st) {
  if (a.T == 0 || a.d == 0) return hipSuccess;
  const dim3 block(kNormWaves * kWave);
  auto aligned = [](const void* p, int64_t ld) { return p == nullptr || (((uintptr_t)p & 15u) == 0 && ld % 8 == 0); };
  const bool fast = a.bf16 && a.d % 8 == 0 && a.d <= 8192 && aligned(a.X, a.ldx) && aligned(a.R, a.ldr) &&
                    aligned(a.Hsum, a.ldh) && aligned(a.Y, a.ldy) && ((uintptr_t)a.gamma & 15u) == 0 &&
                    ((uintptr_t)a.beta & 15u) == 0;
  if (!fast) {
    const dim3 grid((a.T + kNormWaves - 1) / kNormWaves);
    if (a.bf16) k_add_norm_any<bf16_t><<<grid, block, 0, st>>>(a);
    else k_add_norm_any<float><<<grid, block, 0, st>>>(a);
    return hipGetLastError();
  }
  // One round of workgroups: as many as are resident at once (registers and the LDS copy of gamma and
  // beta allow wgs_per_cu per CU), each wave walking through its share of the rows.  More, smaller
  // workgroups re-stage gamma and beta more often and leave a partial last round.
  const int cus = compute_units();
  const int wgs_per_cu = a.d <= 2048 ? 7 : a.d <= 4096 ? 4 : a.d <= 6144 ? 3 : 2;
  const int per_round = cus * wgs_per_cu * kNormWaves;
  const int rows_per_wave = (a.T + per_round - 1) / per_round;
  const int rows_per_wg = rows_per_wave * kNormWaves;
  const dim3 grid((a.T + rows_per_wg - 1) / rows_per_wg);
  if (a.d <= 2048) k_add_norm_bf16<4><<<grid, block, 0, st>>>(a, rows_per_wave);
  else if (a.d <= 4096) k_add_norm_bf16<8><<<grid, block, 0, st>>>(a, rows_per_wave);
  else if (a.d <= 6144) k_add_norm_bf16<12><<<grid, block, 0, st>>>(a, rows_per_wave);
  else k_add_norm_bf16<16><<<grid, block, 0, st>>>(a, rows_per_wave);
  return hipGetLastError();
}

int attention_f32_max_head_dim() { return kAttnF32MaxDh; }
int attention_bf16_head_dim() { return kDh; }

hipError_t launch_attention(const AttnArgs& a, hipStream_t st) {
  if (a.T == 0 || a.S == 0 || a.n_heads == 0) return hipSuccess;
  if (a.bf16) {
    const dim3 grid(((a.T + kBQ - 1) / kBQ + a.S) * a.n_heads);
    k_attention_bf16<<<grid, kAttnWaves * kWave, 0, st>>>(a);
  } else {
    const dim3 grid(a.T, a.n_heads);
    k_attention_f32<<<grid, kWave, 0, st>>>(a);
  }
  return hipGetLastError();
}

}  // namespace zo
