// Schedule planner: Sec. 4.3 (ring of d nodes = d-1 phases of d concurrent transfers of
// 1/d of the data; learners in an m-dimensional box, P = d_1*...*d_m), with the
// reduce-scatter taking dimensions 1..m and the all-gather m..1 (Sec. 4.1 operations).
#include "plan.h"

#include <algorithm>
#include <utility>

namespace ddl {

int dtype_size(ddl_dtype_t dtype) {
    switch (dtype) {
        case DDL_F32: return 4;
        case DDL_F64: return 8;
        case DDL_I32: return 4;
        case DDL_F16: return 2;
        case DDL_BF16: return 2;
    }
    return 0;
}

ddl_status_t validate_dims(const int* dims, int m, int P) {
    if (P < 1 || P > DDL_MAX_LEARNERS) return DDL_ERR_ARG;
    if (dims == nullptr) return DDL_ERR_ARG;
    if (m < 1 || m > DDL_MAX_DIMS) return DDL_ERR_DIMS;
    int64_t prod = 1;
    for (int t = 0; t < m; ++t) {
        if (dims[t] < 1) return DDL_ERR_DIMS;
        prod *= dims[t];
        if (prod > DDL_MAX_LEARNERS) return DDL_ERR_DIMS;
    }
    return prod == P ? DDL_OK : DDL_ERR_DIMS;
}

void split_range(uint64_t lo, uint64_t hi, uint64_t d, uint64_t k, uint64_t G,
                 uint64_t* a, uint64_t* b) {
    const uint64_t n = hi - lo;
    const uint64_t granules = (n + G - 1) / G;
    // d <= 65536 and granules < 2^60: the products cannot overflow
    uint64_t first = (k * granules / d) * G;
    uint64_t last = ((k + 1) * granules / d) * G;
    *a = lo + (first < n ? first : n);
    *b = lo + (last < n ? last : n);
}

void build_schedule(ddl_plan* plan) {
    const int m = static_cast<int>(plan->dims.size());
    const int P = plan->P;
    const int S = static_cast<int>(plan->seg_off.size());
    const uint64_t G = 16 / static_cast<uint64_t>(plan->elem_size);

    std::vector<int> stride(m + 1, 1);  // rank distance of one position along dimension t
    for (int t = 0; t < m; ++t) stride[t + 1] = stride[t] * plan->dims[t];

    // Segment every learner works on at the start of each dimension, per tensor
    // (level 0 = the whole tensor); index [(s * (m + 1) + t) * P + r].
    std::vector<uint64_t> lo(size_t(S) * (m + 1) * P), hi(lo.size());
    auto at = [&](int s, int t, int r) { return (size_t(s) * (m + 1) + t) * P + r; };
    for (int s = 0; s < S; ++s) {
        for (int r = 0; r < P; ++r) {
            lo[at(s, 0, r)] = plan->seg_off[s];
            hi[at(s, 0, r)] = plan->seg_off[s] + plan->seg_count[s];
        }
        for (int t = 0; t < m; ++t) {
            const int d = plan->dims[t];
            for (int r = 0; r < P; ++r) {
                const int pos = (r / stride[t]) % d;
                split_range(lo[at(s, t, r)], hi[at(s, t, r)], d, pos, G, &lo[at(s, t + 1, r)],
                            &hi[at(s, t + 1, r)]);
            }
        }
    }
    plan->own_off.resize(size_t(S) * P);
    plan->own_n.resize(size_t(S) * P);
    for (int s = 0; s < S; ++s)
        for (int r = 0; r < P; ++r) {
            plan->own_off[size_t(s) * P + r] = lo[at(s, m, r)];
            plan->own_n[size_t(s) * P + r] = hi[at(s, m, r)] - lo[at(s, m, r)];
        }

    auto emit = [&](int kind, int t, int phase) {
        const int d = plan->dims[t];
        Step st{kind, t, 0, 0, plan->whole.size(), 0, plan->ragged.size(), 0};
        const uint64_t per_elem = (kind == DDL_STEP_REDUCE ? 3u : 2u) * plan->elem_size;
        for (int s = 0; s < S; ++s) {
            for (int r = 0; r < P; ++r) {
                const int pos = (r / stride[t]) % d;
                const int next = r + ((pos + 1) % d - pos) * stride[t];
                // reduce: in phase s ring position c passes on part c-s-1, the partial sum
                // that set out one position after the part's owner; gather: position c
                // passes on part c-s, its own completed part first.
                const int back = (kind == DDL_STEP_REDUCE) ? phase + 1 : phase;
                const int part = ((pos - back) % d + d) % d;
                Op op;
                split_range(lo[at(s, t, r)], hi[at(s, t, r)], d, part, G, &op.off, &op.n);
                op.n -= op.off;
                op.src = r;
                op.dst = next;
                if (op.n > st.max_n) st.max_n = op.n;
                st.bytes += op.n * per_elem;
                if (S > 1 && op.n > 0) {
                    // work lists for the batched launch (see BlockDesc)
                    const uint64_t nv = op.n / G;                      // whole vectors
                    const uint64_t rows = (nv + 1 + 63 + 63) / 64;     // one more: the shifted tiling
                    const uint32_t index = static_cast<uint32_t>(plan->ops.size());
                    const uint64_t inside = nv / 64;                   // rows [1, inside) are interior
                    uint64_t whole_end = kListHeadRows;
                    if (inside > uint64_t(kListHeadRows))
                        whole_end += (inside - kListHeadRows) / kListRows * kListRows;
                    for (uint64_t row = 0; row < rows && row < uint64_t(kListHeadRows); row += kListTailRows)
                        plan->ragged.push_back(BlockDesc{index, static_cast<uint32_t>(row)});
                    for (uint64_t row = kListHeadRows; row < whole_end; row += kListRows)
                        plan->whole.push_back(BlockDesc{index, static_cast<uint32_t>(row)});
                    for (uint64_t row = whole_end; row < rows; row += kListTailRows)
                        plan->ragged.push_back(BlockDesc{index, static_cast<uint32_t>(row)});
                }
                plan->ops.push_back(op);
            }
        }
        st.whole_count = plan->whole.size() - st.whole_first;
        st.ragged_count = plan->ragged.size() - st.ragged_first;
        plan->bytes_total += st.bytes;
        plan->steps.push_back(st);
    };

    for (int t = 0; t < m; ++t)
        for (int phase = 0; phase + 1 < plan->dims[t]; ++phase) emit(DDL_STEP_REDUCE, t, phase);
    plan->first_gather = static_cast<int>(plan->steps.size());
    for (int t = m - 1; t >= 0; --t)
        for (int phase = 0; phase + 1 < plan->dims[t]; ++phase) emit(DDL_STEP_GATHER, t, phase);
}

ddl_status_t verify_plan(const ddl_plan& plan) {
    const int P = plan.P;
    const size_t S = plan.seg_off.size();
    const uint64_t G = 16 / uint64_t(plan.elem_size);
    const size_t per_step = S * size_t(P);
    if (plan.ops.size() != plan.steps.size() * per_step) return DDL_ERR_ARG;
    std::vector<int> stride(plan.dims.size() + 1, 1);
    for (size_t t = 0; t < plan.dims.size(); ++t) stride[t + 1] = stride[t] * plan.dims[t];
    std::vector<int> received(P);
    for (size_t s = 0; s < plan.steps.size(); ++s) {
        const Step& st = plan.steps[s];
        if (st.dim < 0 || st.dim >= int(plan.dims.size())) return DDL_ERR_ARG;
        const int d = plan.dims[st.dim];
        for (size_t seg = 0; seg < S; ++seg) {
            const Op* ops = plan.ops.data() + s * per_step + seg * P;
            std::fill(received.begin(), received.end(), -1);
            for (int r = 0; r < P; ++r) {
                const Op& op = ops[r];
                if (op.src != r || op.dst < 0 || op.dst >= P || received[op.dst] != -1) return DDL_ERR_ARG;
                received[op.dst] = r;
                // the receiver is the next position on the sender's ring of this dimension
                const int pos = (r / stride[st.dim]) % d;
                if (op.dst != r + ((pos + 1) % d - pos) * stride[st.dim]) return DDL_ERR_ARG;
                if (op.off < plan.seg_off[seg] || op.off + op.n > plan.seg_off[seg] + plan.seg_count[seg])
                    return DDL_ERR_ARG;
                if (op.n > 0 && (op.off - plan.seg_off[seg]) % G != 0) return DDL_ERR_ARG;
            }
            for (int r = 0; r < P; ++r) {
                // what learner r receives must not touch what it sends
                const Op& out = ops[r];
                const Op& in = ops[received[r]];
                if (in.n > 0 && out.n > 0 && in.off < out.off + out.n && out.off < in.off + in.n) return DDL_ERR_ARG;
            }
        }
    }
    // finest chunks: along every ring of the last dimension... simply: all P chunks of a tensor,
    // sorted by offset, tile it
    for (size_t seg = 0; seg < S; ++seg) {
        std::vector<std::pair<uint64_t, uint64_t>> chunks;
        for (int r = 0; r < P; ++r)
            chunks.emplace_back(plan.own_off[seg * P + r], plan.own_n[seg * P + r]);
        std::sort(chunks.begin(), chunks.end());
        uint64_t at = plan.seg_off[seg];
        for (const auto& c : chunks) {
            if (c.second == 0) continue;
            if (c.first != at) return DDL_ERR_ARG;
            at += c.second;
        }
        if (at != plan.seg_off[seg] + plan.seg_count[seg]) return DDL_ERR_ARG;
    }
    for (const WalkLevel& lv : plan.walk_levels)
        for (int half = 0; half < 2; ++half) {
            for (size_t r = 0; r < S * size_t(P); ++r) {
                const uint64_t* row = plan.walk_plan.data() + (half ? lv.gather_plan : lv.reduce_plan) +
                                      r * (size_t(lv.d) + 2);
                const size_t seg = r / P;
                if (row[0] < plan.seg_off[seg] || row[0] + row[1] > plan.seg_off[seg] + plan.seg_count[seg] ||
                    row[2] != uint64_t(r % P))
                    return DDL_ERR_ARG;
                for (int i = 0; i + 1 < lv.d; ++i) {
                    const int a = int(row[2 + i]);
                    const int pos = (a / stride[lv.dim]) % lv.d;
                    if (int(row[3 + i]) != a + ((pos + 1) % lv.d - pos) * stride[lv.dim]) return DDL_ERR_ARG;
                }
            }
            // several tensors: every tile of every non-empty row listed once, in order
            if (S > 1) {
                const BlockDesc* item = plan.walk_items.data() + (half ? lv.gather_items : lv.reduce_items);
                const BlockDesc* end = item + (half ? lv.gather_count : lv.reduce_count);
                for (size_t r = 0; r < S * size_t(P); ++r) {
                    const uint64_t n = plan.walk_plan[(half ? lv.gather_plan : lv.reduce_plan) + r * (size_t(lv.d) + 2) + 1];
                    if (n == 0) continue;
                    const uint64_t tile_vecs = uint64_t(kWalkListRows) * 64;
                    const uint64_t tiles = (n / G + 1 + 63 + tile_vecs - 1) / tile_vecs;
                    for (uint64_t tile = 0; tile < tiles; ++tile, ++item)
                        if (item >= end || item->op != r || item->row != tile) return DDL_ERR_ARG;
                }
                if (item != end) return DDL_ERR_ARG;
            }
        }
    return DDL_OK;
}

void build_walk(ddl_plan* plan) {
    plan->walk_levels.clear();
    plan->walk_plan.clear();
    plan->walk_items.clear();
    plan->walk_words = 0;
    plan->walk_bytes = 0;
    if (plan->steps.empty()) return;
    const int P = plan->P;
    const size_t S = plan->seg_off.size();
    const size_t rows = S * size_t(P);
    const uint64_t G = 16 / uint64_t(plan->elem_size);
    size_t words = 0;
    for (int d : plan->dims)
        if (d > 1) words += 2 * rows * (size_t(d) + 2);
    if (words > kWalkMaxWords) return;
    // first phase of every dimension's reduce-scatter and all-gather in the step list
    std::vector<int> first_reduce(plan->dims.size(), -1), first_gather(plan->dims.size(), -1);
    for (int s = static_cast<int>(plan->steps.size()) - 1; s >= 0; --s) {
        const Step& st = plan->steps[s];
        (st.kind == DDL_STEP_REDUCE ? first_reduce : first_gather)[st.dim] = s;
    }
    int last = -1;
    for (size_t u = 0; u < plan->dims.size(); ++u)
        if (plan->dims[u] > 1) last = int(u);
    for (size_t t = 0; t < plan->dims.size(); ++t) {
        const int d = plan->dims[t];
        if (d <= 1) continue;
        WalkLevel level{int(t), d, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        for (int half = 0; half < 2; ++half) {
            const int s0 = half == 0 ? first_reduce[t] : first_gather[t];
            (half == 0 ? level.reduce_plan : level.gather_plan) = plan->walk_plan.size();
            (half == 0 ? level.reduce_rows : level.gather_rows) = plan->walk_words;
            (half == 0 ? level.reduce_items : level.gather_items) = plan->walk_items.size();
            plan->walk_words += rows * (size_t(d) + 1);
            for (size_t row = 0; row < rows; ++row) {
                // the chunk that learner r passes on in the dimension's first phase keeps its
                // range through all d-1 phases; its path is r, next(r), next(next(r)), ...
                const size_t seg = row / P;
                const Op& op0 = plan->ops[size_t(s0) * rows + row];
                plan->walk_plan.push_back(op0.off);
                plan->walk_plan.push_back(op0.n);
                int at = int(row % P);
                for (int i = 0; i < d; ++i) {
                    plan->walk_plan.push_back(uint64_t(at));
                    if (i + 1 < d) at = plan->ops[size_t(s0 + i) * rows + seg * P + at].dst;
                }
                if (op0.n > level.max_n) level.max_n = op0.n;
                // reduce: d reads and d-1 writes of the chunk; gather: 1 read and d-1 writes;
                // the last dimension of the allreduce does both at once: d reads, d writes
                const int accesses = int(t) == last ? (half == 0 ? 2 * d : 0) : (half == 0 ? 2 * d - 1 : d);
                plan->walk_bytes += op0.n * uint64_t(plan->elem_size) * uint64_t(accesses);
                if (S > 1 && op0.n > 0) {
                    // tiles of kWalkListRows rows; one row more than the vectors need, because
                    // the tiling is shifted onto absolute row boundaries at run time
                    const uint64_t tile_vecs = uint64_t(kWalkListRows) * 64;
                    const uint64_t tiles = (op0.n / G + 1 + 63 + tile_vecs - 1) / tile_vecs;
                    for (uint64_t tile = 0; tile < tiles; ++tile)
                        plan->walk_items.push_back(BlockDesc{uint32_t(row), uint32_t(tile)});
                }
            }
            (half == 0 ? level.reduce_count : level.gather_count) =
                plan->walk_items.size() - (half == 0 ? level.reduce_items : level.gather_items);
        }
        plan->walk_levels.push_back(level);
    }
}

int build_fused_order(const ddl_plan& plan, std::vector<uint32_t>* seq, std::vector<uint32_t>* ctl,
                      int* padded) {
    // Rings of size 1 add nothing; the others are the levels, dimension 1 innermost.
    std::vector<int> size, stride;
    int s = 1;
    for (int d : plan.dims) {
        if (d > 1) {
            size.push_back(d);
            stride.push_back(s);
        }
        s *= d;
    }
    const int levels = static_cast<int>(size.size());
    const int P = plan.P;
    const int pad = (P + kFusedBatch - 1) / kFusedBatch * kFusedBatch;
    *padded = pad;
    seq->assign(size_t(P) * pad, 0);
    ctl->assign(pad, 0);
    std::vector<int> digit(levels, 0);
    for (int i = 0; i < P; ++i) {
        // item i = mixed-radix digits (i_1 fastest): position k_t + 1 + i_t on the ring of level t
        uint32_t word = kFusedValid;
        for (int t = 0; t < levels; ++t) {
            if (digit[t] == 0) word |= 1u << t;
            if (digit[t] == size[t] - 1) word |= 1u << (8 + t);
        }
        (*ctl)[i] = word;
        for (int c = 0; c < P; ++c) {
            int rank = 0;
            for (int t = 0; t < levels; ++t) {
                const int k = (c / stride[t]) % size[t];
                rank += ((k + 1 + digit[t]) % size[t]) * stride[t];
            }
            (*seq)[size_t(c) * pad + i] = static_cast<uint32_t>(rank);
        }
        for (int t = 0; t < levels; ++t) {
            if (++digit[t] < size[t]) break;
            digit[t] = 0;
        }
    }
    for (int c = 0; c < P; ++c)
        for (int i = P; i < pad; ++i) (*seq)[size_t(c) * pad + i] = (*seq)[size_t(c) * pad];
    return levels;
}

double model_time(const int* dims, int m, double bytes, const double* bw, const double* lat) {
    double level_bytes = bytes;
    double total = 0.0;
    for (int t = 0; t < m; ++t) {
        const int d = dims[t];
        total += 2.0 * (d - 1) * (level_bytes / (d * bw[t]) + lat[t]);
        level_bytes /= d;
    }
    return total;
}

namespace {

struct Search {
    int P, m;
    double bytes;
    const double *bw, *lat;
    const int* max_dim;
    std::vector<int> cur, best;
    double best_time = -1.0;

    void visit(int t, int remaining) {
        if (t == m - 1) {
            if (max_dim && max_dim[t] > 0 && remaining > max_dim[t]) return;
            cur[t] = remaining;
            const double time = model_time(cur.data(), m, bytes, bw, lat);
            // enumeration is in lexicographic order, so "<" keeps the first of equal scores
            if (best_time < 0.0 || time < best_time) {
                best_time = time;
                best = cur;
            }
            return;
        }
        for (int d = 1; d <= remaining; ++d) {
            if (remaining % d != 0) continue;
            if (max_dim && max_dim[t] > 0 && d > max_dim[t]) break;
            cur[t] = d;
            visit(t + 1, remaining / d);
        }
    }
};

}  // namespace

ddl_status_t choose_dims(int P, double bytes, int m, const double* bw, const double* lat,
                         const int* max_dim, int* dims_out, double* time_out) {
    if (P < 1 || P > DDL_MAX_LEARNERS || bw == nullptr || lat == nullptr || dims_out == nullptr)
        return DDL_ERR_ARG;
    if (m < 1 || m > DDL_MAX_DIMS) return DDL_ERR_DIMS;
    for (int t = 0; t < m; ++t)
        if (!(bw[t] > 0.0) || !(lat[t] >= 0.0) || (max_dim && max_dim[t] < 0)) return DDL_ERR_ARG;
    Search s{P, m, bytes, bw, lat, max_dim, std::vector<int>(m, 1), {}, -1.0};
    s.visit(0, P);
    if (s.best.empty()) return DDL_ERR_DIMS;
    for (int t = 0; t < m; ++t) dims_out[t] = s.best[t];
    if (time_out) *time_out = s.best_time;
    return DDL_OK;
}

}  // namespace ddl
