// Fused candidate scoring: s(q,e) = gamma - min_b ||y_b - E[e]||_1 for the
// positive and the K negatives of every query, the log-sigmoid loss terms,
// dL/ds per pair and the gradient of every branch embedding, in one pass over
// the candidate rows (Sec. 4.2 "Vectorized Logit Formulation": all positive and
// negative candidates of the batch are scored together; the entity rows are
// fetched through precomputed ids and never materialised).
//
// One workgroup per query; each wavefront streams whole candidate rows (a lane
// holds float4 pieces 64 apart, so a row is read in fully coalesced 1 KB
// requests), reduces |y - e| across the wavefront, and keeps its share of
// dL/dy in registers (one branch) or LDS (union queries).  Partial sums of the
// wavefronts are combined in a fixed order, so results do not depend on timing.
#include "common.h"

namespace ngdb {
namespace {

__device__ __forceinline__ uint32_t sign_code(float s) { return s > 0.f ? 1u : (s < 0.f ? 2u : 0u); }
__device__ __forceinline__ int32_t cand_id(const ScoreArgs& a, int i, int has_pos, int c) {
    return (has_pos && c == 0) ? a.pos[i] : a.cand[(size_t)i * a.C + (c - has_pos)];
}
// The float4 piece of a row that lane holds in its register chunk ch.  fp32 rows: pieces 64
// apart (a wavefront reads 1 KB per request).  bf16 rows (B16; two chunks per 16-byte load): a
// lane owns 8 consecutive coordinates, so that a request again covers 1 KB of contiguous row.
template <bool B16>
__device__ __forceinline__ int col_of(int ch, int lane) {
    return B16 ? (ch >> 1) * 128 + 2 * lane + (ch & 1) : ch * 64 + lane;
}
typedef uint32_t score_u32x4 __attribute__((ext_vector_type(4)));
template <int NCH, bool B16>
__device__ __forceinline__ void load_row(const ScoreArgs& a, int32_t e, int lane, int d4, float4 (&dst)[NCH]) {
    if (B16) {   // the bf16 copy of the table: 16 bytes (8 coordinates) per lane and chunk pair; d % 8 == 0
        const score_u32x4* row = reinterpret_cast<const score_u32x4*>(a.E16 + (size_t)e * a.d);
        const int d8 = d4 >> 1;
#pragma unroll
        for (int g = 0; g < NCH / 2; ++g) {
            const score_u32x4 v = row[min(g * 64 + lane, d8 - 1)];
            dst[2 * g] = bf16x4_to_f32(make_uint2(v[0], v[1]));
            dst[2 * g + 1] = bf16x4_to_f32(make_uint2(v[2], v[3]));
        }
    } else {
        const float4* row = reinterpret_cast<const float4*>(a.E + (size_t)e * a.d);
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) dst[ch] = row[min(ch * 64 + lane, d4 - 1)];
    }
}

// MASK (training with text features): sign codes per pair instead of the winning rows.
// BOX: the query side is a box (centre from act, offset from off) and the distance is
// sum relu(|e-c| - o) + alpha * sum min(|e-c|, o); in LDS the offsets of the branches follow
// the centres and the offset gradients follow the centre gradients.
// Gradients of the query side: a wavefront keeps those of branch 0 in registers and those of the
// other branches (unions) in LDS accumulators of its own.  At the end the registers are summed
// over the wavefronts: in workgroups of four wavefronts (large batches, where occupancy decides)
// one after the other into the LDS area that held the branch rows, so that LDS per workgroup
// stays small enough for eight wavefronts per SIMD; in larger workgroups (small batches) through
// a staging area per wavefront and one barrier.
// B16: candidate rows come from the bf16 copy of the table.
// STASH: the per-pair results (score, dL/ds, winning branch) are kept in LDS and written after the
// candidate loop.  Stores under a lane condition inside the loop would make every wait in it a wait
// for everything outstanding (the compiler cannot count requests that may or may not be issued),
// the row requested ahead included.
template <int NCH, int NW, bool TRAIN, bool MASK, bool BOX, bool B16, bool STASH>
__global__ __launch_bounds__(NW * 64) void score_kernel(const ScoreArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int i = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int d4 = a.d >> 2;
    const int r0 = a.root_off[i];
    const int nb = a.root_off[i + 1] - r0;
    const int has_pos = a.pos ? 1 : 0;
    const int CT = a.C + has_pos;

    constexpr int PARTS = BOX ? 2 : 1;                               // centre (and offset) per branch
    float4* ybr = reinterpret_cast<float4*>(lds);                    // [PARTS][nb][d4]
    float4* accs = ybr + (size_t)PARTS * a.max_branch * d4;          // [NW][PARTS][nb-1][d4]   (TRAIN)
    constexpr bool SEQ = NW <= 4;                                    // how branch 0 is summed over the wavefronts
    float4* stage = accs + (TRAIN ? (size_t)NW * PARTS * (a.max_branch - 1) * d4 : 0);   // [NW][PARTS][d4]  (!SEQ)
    float* lossp = reinterpret_cast<float*>(stage + (TRAIN && !SEQ ? (size_t)NW * PARTS * d4 : 0));
    float* out_s = lossp + 16;                                       // [CT] scores          (STASH)
    float* out_c = out_s + CT;                                       // [CT] dL/ds           (STASH, TRAIN)
    int* out_b = reinterpret_cast<int*>(out_c + CT);                 // [CT] winning branch  (STASH, TRAIN, no MASK)
    const float4* obr = ybr + (size_t)nb * d4;                       // offsets (BOX)

    for (int idx = tid; idx < PARTS * nb * d4; idx += NW * 64) {
        const int b = idx / d4, c = idx - b * d4;
        const float* src = (BOX && b >= nb) ? a.off + (size_t)a.root_slot[r0 + b - nb] * a.d
                                            : a.act + (size_t)a.root_slot[r0 + b] * a.d;
        ybr[idx] = reinterpret_cast<const float4*>(src)[c];
    }
    const int nx = nb - 1;                                           // branches kept in LDS
    float4* myacc = accs + (size_t)wave * PARTS * nx * d4;           // [PARTS][nx][d4]
    if (TRAIN)
        for (int idx = lane; idx < PARTS * nx * d4; idx += 64) myacc[idx] = make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();

    const float inv2B = 1.f / (2.f * (float)a.B);
    const float invK = a.C > 0 ? 1.f / (float)a.C : 0.f;
    float4 dyr[NCH], dor[BOX ? NCH : 1];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
        dyr[ch] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (BOX) dor[ch] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    const float alpha = a.alpha;
    float lsum = 0.f;

    // The id of a candidate is requested two rounds ahead of its use and its row one round
    // ahead, so that a row request never waits for its id (more rows in flight per wavefront,
    // three sets of row registers used in turn, gain 1 % on long candidate lists and lose 20 %
    // on short ones).  Requests past the end repeat the last candidate (clamped, no branches
    // around loads).
    float4 cur[NCH], nxt[NCH];
    int c = wave;
    int32_t e_nxt = cand_id(a, i, has_pos, min(c + NW, CT - 1));
    if (c < CT) load_row<NCH, B16>(a, cand_id(a, i, has_pos, c), lane, d4, cur);
    for (; c < CT; c += NW) {
        load_row<NCH, B16>(a, e_nxt, lane, d4, nxt);
        e_nxt = cand_id(a, i, has_pos, min(c + 2 * NW, CT - 1));
        float best = INFINITY;
        int bw = 0;
        for (int b = 0; b < nb; ++b) {
            float dist = 0.f;
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                const int col = col_of<B16>(ch, lane);
                if (col < d4) {
                    const float4 y = ybr[b * d4 + col];
                    const float ax = fabsf(y.x - cur[ch].x), ay = fabsf(y.y - cur[ch].y),
                                az = fabsf(y.z - cur[ch].z), aw = fabsf(y.w - cur[ch].w);
                    if (BOX) {
                        const float4 o = obr[b * d4 + col];
                        dist += ((fmaxf(ax - o.x, 0.f) + fmaxf(ay - o.y, 0.f)) +
                                 (fmaxf(az - o.z, 0.f) + fmaxf(aw - o.w, 0.f))) +
                                alpha * ((fminf(ax, o.x) + fminf(ay, o.y)) + (fminf(az, o.z) + fminf(aw, o.w)));
                    } else {
                        dist += (ax + ay) + (az + aw);
                    }
                }
            }
            dist = wave_sum_dpp(dist);
            if (dist < best) {   // strict: equal distances keep the lower branch
                best = dist;
                bw = b;
            }
        }
        const float s = a.gamma - best;
        const size_t pair = (size_t)i * CT + c;
        if (STASH) out_s[c] = s;                 // (every lane the same value to the same word)
        else if (lane == 0) a.score[pair] = s;
        if (TRAIN) {
            const bool is_pos = (c == 0);
            // The positive contributes softplus(-s) with dL/ds = -sigmoid(-s)/(2B), a negative
            // softplus(s)/K with dL/ds = sigmoid(s)/(2BK): with z = -s resp. s both are
            // w * softplus(z) and +-w * sigmoid(z) / (2B).  One exponential serves both: with
            // e = exp(-|z|), sigmoid(z) = 1/(1+e) or e/(1+e), softplus(z) = max(z, 0) + log(1+e).
            // The hardware approximations (about 1 ulp, the argument of the exponential rounded
            // once) keep dL/ds to a few 1e-6 relative; the correctly rounded library forms cost
            // several hundred instructions per pair, every one of them on all 64 lanes.
            const float z = is_pos ? -s : s;
            const float wq = is_pos ? 1.f : invK;
            const float e = fast_exp_neg(fabsf(z));
            const float r = fast_rcp(1.f + e);
            const float sig = z >= 0.f ? r : e * r;
            const float coef = (is_pos ? -inv2B : inv2B) * wq * sig;
            lsum += wq * (fmaxf(z, 0.f) + fast_log1p_unit(e));
            if (STASH) {
                out_c[c] = coef;
                if (!MASK) out_b[c] = bw;
            } else if (lane == 0) {
                a.coef[pair] = coef;
                if (!MASK) a.win[pair] = a.root_slot[r0 + bw];
            }
            uint32_t bits = 0;      // 2 bits per coordinate of this lane: 1 = positive, 2 = negative difference
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                const int col = col_of<B16>(ch, lane);
                if (col < d4) {
                    const float4 y = ybr[bw * d4 + col];
                    const float tx = y.x - cur[ch].x, ty = y.y - cur[ch].y, tz = y.z - cur[ch].z, tw = y.w - cur[ch].w;
                    if (MASK)
                        bits |= (sign_code(tx) | (sign_code(ty) << 2) | (sign_code(tz) << 4) | (sign_code(tw) << 6)) << (8 * ch);
                    float4 g;                                     // coef * sign(difference)
                    g.x = signed_by(coef, tx);
                    g.y = signed_by(coef, ty);
                    g.z = signed_by(coef, tz);
                    g.w = signed_by(coef, tw);
                    if (BOX) {
                        // outside coordinates pull the centre with weight 1 and widen the offset;
                        // inside ones pull with weight alpha and leave the offset alone
                        const float4 o = obr[bw * d4 + col];
                        const bool ox = fabsf(tx) > o.x, oy = fabsf(ty) > o.y, oz = fabsf(tz) > o.z, ow = fabsf(tw) > o.w;
                        g.x *= ox ? 1.f : alpha; g.y *= oy ? 1.f : alpha;
                        g.z *= oz ? 1.f : alpha; g.w *= ow ? 1.f : alpha;
                        const float co = coef * (1.f - alpha);
                        float4 go;
                        go.x = ox ? co : 0.f; go.y = oy ? co : 0.f; go.z = oz ? co : 0.f; go.w = ow ? co : 0.f;
                        if (bw == 0) {
                            dor[ch].x += go.x; dor[ch].y += go.y; dor[ch].z += go.z; dor[ch].w += go.w;
                        } else {
                            float4 t = myacc[(nx + bw - 1) * d4 + col];
                            t.x += go.x; t.y += go.y; t.z += go.z; t.w += go.w;
                            myacc[(nx + bw - 1) * d4 + col] = t;
                        }
                    }
                    if (bw == 0) {
                        dyr[ch].x -= g.x; dyr[ch].y -= g.y; dyr[ch].z -= g.z; dyr[ch].w -= g.w;
                    } else {
                        float4 t = myacc[(bw - 1) * d4 + col];
                        t.x -= g.x; t.y -= g.y; t.z -= g.z; t.w -= g.w;
                        myacc[(bw - 1) * d4 + col] = t;
                    }
                }
            }
            // text features: the signs of the pair, from which the table pass rebuilds coef * sign
            // (the scored row is not the table row there)
            if (MASK) {
                if (NCH == 1) reinterpret_cast<uint8_t*>(a.mask)[pair * 64 + lane] = (uint8_t)bits;
                else if (NCH == 2) reinterpret_cast<uint16_t*>(a.mask)[pair * 64 + lane] = (uint16_t)bits;
                else reinterpret_cast<uint32_t*>(a.mask)[pair * 64 + lane] = bits;
            }
        }
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) cur[ch] = nxt[ch];
    }

    if (STASH) {
        __syncthreads();
        for (int idx = tid; idx < CT; idx += NW * 64) {
            const size_t pair = (size_t)i * CT + idx;
            a.score[pair] = out_s[idx];
            if (TRAIN) {
                a.coef[pair] = out_c[idx];
                if (!MASK) a.win[pair] = a.root_slot[r0 + out_b[idx]];
            }
        }
    }
    if (TRAIN) {
        if (lane == 0) lossp[wave] = lsum;
        // branch 0: summed over the wavefronts in a fixed order, either through the staging area or
        // in turn into the area of the branch rows, which nobody reads any more after the first barrier
        float4* red = ybr;                                           // [PARTS][d4]  (SEQ)
        const int root0 = a.root_slot[r0];
        if (!SEQ) {
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                const int col = col_of<B16>(ch, lane);
                if (col < d4) {
                    stage[(size_t)wave * PARTS * d4 + col] = dyr[ch];
                    if (BOX) stage[(size_t)wave * PARTS * d4 + d4 + col] = dor[ch];
                }
            }
            __syncthreads();
            for (int idx = tid; idx < PARTS * d4; idx += NW * 64) {
                float4 t = stage[idx];
                for (int w = 1; w < NW; ++w) {
                    const float4 u = stage[(size_t)w * PARTS * d4 + idx];
                    t.x += u.x; t.y += u.y; t.z += u.z; t.w += u.w;
                }
                const int part = idx / d4, cc = idx - part * d4;
                reinterpret_cast<float4*>((part ? a.doff : a.dact) + (size_t)root0 * a.d)[cc] = t;
            }
        }
        for (int w = 0; SEQ && w < NW; ++w) {
            __syncthreads();
            if (wave == w) {
#pragma unroll
                for (int ch = 0; ch < NCH; ++ch) {
                    const int col = col_of<B16>(ch, lane);
                    if (col < d4) {
                        float4 t = dyr[ch];
                        if (w > 0) {
                            const float4 u = red[col];
                            t.x += u.x; t.y += u.y; t.z += u.z; t.w += u.w;
                        }
                        red[col] = t;
                        if (BOX) {
                            float4 q = dor[ch];
                            if (w > 0) {
                                const float4 u = red[d4 + col];
                                q.x += u.x; q.y += u.y; q.z += u.z; q.w += u.w;
                            }
                            red[d4 + col] = q;
                        }
                    }
                }
            }
        }
        __syncthreads();
        for (int idx = tid; SEQ && idx < PARTS * d4; idx += NW * 64) {
            const int part = idx / d4, cc = idx - part * d4;
            float* dst = (part ? a.doff : a.dact) + (size_t)root0 * a.d;
            reinterpret_cast<float4*>(dst)[cc] = red[idx];
        }
        // the other branches: sum of the wavefronts' LDS accumulators
        for (int idx = tid; idx < PARTS * nx * d4; idx += NW * 64) {
            float4 t = accs[idx];
            for (int w = 1; w < NW; ++w) {
                const float4 u = accs[(size_t)w * PARTS * nx * d4 + idx];
                t.x += u.x; t.y += u.y; t.z += u.z; t.w += u.w;
            }
            const int b = idx / d4, cc = idx - b * d4;              // b over [PARTS][nx]
            float* dst = (BOX && b >= nx) ? a.doff + (size_t)a.root_slot[r0 + 1 + b - nx] * a.d
                                          : a.dact + (size_t)a.root_slot[r0 + 1 + b] * a.d;
            reinterpret_cast<float4*>(dst)[cc] = t;
        }
        if (tid == 0) {
            float l = 0.f;
            for (int w = 0; w < NW; ++w) l += lossp[w];
            a.loss_terms[i] = l;
        }
    }
}

constexpr int STASH_MAX_PAIRS = 4096;     // pairs per query whose results fit the LDS stash (48 KB)
template <int NCH, int NW, bool TRAIN, bool MASK, bool BOX, bool B16, bool STASH>
hipError_t launch_stash(const ScoreArgs& a, size_t lds, hipStream_t s) {
    if (lds > 64 * 1024)
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(score_kernel<NCH, NW, TRAIN, MASK, BOX, B16, STASH>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL((score_kernel<NCH, NW, TRAIN, MASK, BOX, B16, STASH>), dim3(a.B), dim3(NW * 64), lds, s, a);
    return hipGetLastError();
}
template <int NCH, int NW, bool TRAIN, bool MASK, bool BOX, bool B16 = false>
hipError_t launch_variant(const ScoreArgs& a, size_t lds, hipStream_t s) {
    const int CT = a.C + (a.pos ? 1 : 0);
    const size_t stash = (size_t)CT * (TRAIN ? 3 : 1) * sizeof(float);
    if (CT <= STASH_MAX_PAIRS && lds + stash <= 150 * 1024)
        return launch_stash<NCH, NW, TRAIN, MASK, BOX, B16, true>(a, lds + stash, s);
    return launch_stash<NCH, NW, TRAIN, MASK, BOX, B16, false>(a, lds, s);
}

template <int NCH, int NW>
hipError_t launch_nw(const ScoreArgs& a, bool train, size_t lds, hipStream_t s) {
    if (a.off) return train ? launch_variant<NCH, NW, true, false, true>(a, lds, s)
                            : launch_variant<NCH, NW, false, false, true>(a, lds, s);
    if (a.E16) return train ? launch_variant<NCH, NW, true, false, false, true>(a, lds, s)
                            : launch_variant<NCH, NW, false, false, false, true>(a, lds, s);
    if (train && a.mask) return launch_variant<NCH, NW, true, true, false>(a, lds, s);
    if (train) return launch_variant<NCH, NW, true, false, false>(a, lds, s);
    return launch_variant<NCH, NW, false, false, false>(a, lds, s);
}

template <int NCH>
hipError_t launch_nch(const ScoreArgs& a, bool train, hipStream_t s) {
    // enough wavefronts to cover the chip even for small batches
    const int nw = a.B >= 2048 ? 4 : (a.B >= 1024 ? 8 : 16);
    auto lds_for = [&](int w) {
        const int per_wave = a.max_branch - 1 + (w <= 4 ? 0 : 1);   // union accumulators (+ staging)
        return ((size_t)(a.off ? 2 : 1) * a.d * (a.max_branch + (train ? w * per_wave : 0)) + 16) * sizeof(float);
    };
    const size_t cap = 150 * 1024;
    if (nw == 16 && lds_for(16) <= cap) return launch_nw<NCH, 16>(a, train, lds_for(16), s);
    if (nw >= 8 && lds_for(8) <= cap) return launch_nw<NCH, 8>(a, train, lds_for(8), s);
    if (lds_for(4) <= cap) return launch_nw<NCH, 4>(a, train, lds_for(4), s);
    return hipErrorInvalidValue;   // too many union branches for this width
}

}  // namespace

hipError_t launch_score(const ScoreArgs& a, bool train, hipStream_t s) {
    if (a.B <= 0) return hipSuccess;
    if (a.C + (a.pos ? 1 : 0) <= 0) return hipErrorInvalidValue;   // the kernel clamps into a non-empty candidate list
    if (train && (a.win == nullptr) == (a.mask == nullptr)) return hipErrorInvalidValue;   // exactly one of the two
    if (a.off && (a.mask || (train && !a.doff))) return hipErrorInvalidValue;
    if (a.E16 && (a.off || a.mask)) return hipErrorInvalidValue;     // plain vector family only
    if (a.E16 && (a.d & 7)) return hipErrorInvalidValue;            // 16-byte loads of bf16 rows
    if (a.d <= 256 && !a.E16) return launch_nch<1>(a, train, s);    // (bf16 rows: chunks come in pairs)
    if (a.d <= 512) return launch_nch<2>(a, train, s);
    if (a.d <= 1024) return launch_nch<4>(a, train, s);
    return hipErrorInvalidValue;
}

}  // namespace ngdb
