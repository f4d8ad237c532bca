// Host-only part of the library: Alg. 4 "init" (drawing the hash constants from the seed),
// the per-row traversal plan, and status strings.  No GPU is touched here.
#include <stdint.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "csketch.h"

namespace {

constexpr uint64_t kP61 = (1ull << 61) - 1;
typedef unsigned __int128 u128;

// The traversal plans are found by scanning candidate strides / offsets one by one (about a
// nanosecond each).  The scans stop here, so that cs_params_init returns in seconds whatever
// d_hint is: a longer vector gets the best stride below the cap and no visit list.
constexpr uint64_t kPlanScanMax = 1ull << 28;

// SplitMix64 (Steele, Lea, Flood 2014): the generator that the hash constants are drawn from.
uint64_t splitmix64(uint64_t* s) {
    uint64_t z = (*s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

uint64_t mulmod(uint64_t a, uint64_t b) { return (uint64_t)(((u128)a * b) % kP61); }

// Lane stride for one row.
//
// Along coordinates i, i + D, i + 2D, ... the hash value moves by AD = a*D mod p each time,
// and the bucket (value mod c; c | 2^61 so p = -1 mod c) by (AD mod c), plus 1 whenever the
// value wraps past p: on average by  sigma(D) = (AD mod c) + AD / p  buckets, read as a signed
// number in (-c/2, c/2].  A group of L lanes taking coordinates D apart touches a stretch of
// about L |sigma| cells; a wavefront holds 64 / L groups, so it sends about
// 4 |sigma| + 64 / L requests of 64 bytes.  A super-tile is L D coordinates, so lanes idle
// when L D does not divide into the vector length d.  A wavefront step costs about as much
// instruction issue as one request costs the atomic unit (measured), so the plan minimises
// (1 + requests per wavefront) x (idle-lane overhead) over all D and L in {16, 32, 64} by
// brute force: one 64-bit add per candidate D, once per sketch.
void plan_row(cs_row_plan* rp, uint64_t a, uint64_t as, uint32_t c, bool pow2, uint64_t d_hint) {
    uint64_t best_D = 1;
    int best_L = 64;
    if (pow2 && c >= 64) {
        const uint64_t d_eff = d_hint ? d_hint : 64ull * c;
        uint64_t d_max = d_eff / 8;                     // at least 8 lanes busy
        if (d_max > 16ull * c) d_max = 16ull * c;
        double best_cost = 1e300;
        uint64_t x = 0;                                 // (a * D) mod p
        const double inv_p = 1.0 / (double)kP61;
        for (uint64_t D = 1; D <= d_max; ++D) {
            x += a;
            if (x >= kP61) x -= kP61;
            double adv = (double)(x & (c - 1)) + (double)x * inv_p;   // [0, c + 1)
            if (adv > 0.5 * c) adv -= (double)c;
            if (adv < 0) adv = -adv;
            if (adv > 8.0) continue;                    // more than ~33 requests: never chosen
            for (int L = 16; L <= 64; L *= 2) {
                const double req = 4.0 * adv + 64.0 / L;
                const uint64_t span = (uint64_t)L * D;
                const double waste = (double)(((d_eff + span - 1) / span) * span) / (double)d_eff;
                const double cost = (1.0 + req) * waste;
                if (cost < best_cost) { best_cost = cost; best_D = D; best_L = L; }
            }
        }
    }
    rp->lanes = best_L;
    rp->D = best_D;
    rp->AD = mulmod(a, rp->D);
    rp->ADs = mulmod(as, rp->D);
    // Longest run of neighbouring lanes in one bucket.  Rotating a hash value left by
    // lg(2^61 / c) bits (a multiplication by 2^61 / c mod p) moves the bucket bits to the top, so
    // the bucket is the position on a circle of circumference p cut into arcs of 2^61 / c, and a
    // lane step moves that position by exactly Au = (AD * 2^61 / c) mod p.  At most
    // floor((arc - 1) / min(Au, p - Au)) + 1 consecutive positions fit into one arc.
    rp->scan_steps = 4;
    if (pow2) {
        const uint64_t arc = (1ull << 61) / c;
        const uint64_t Au = mulmod(rp->AD, arc % kP61);
        const uint64_t A1 = Au < kP61 - Au ? Au : kP61 - Au;
        if (A1 > 0) {
            const uint64_t longest = (arc - 1) / A1 + 1;
            int steps = 0;
            while (steps < 4 && (1ull << steps) < longest) ++steps;
            rp->scan_steps = steps;
        }
    }
}

// Walk stride of the update for one row.
//
// A lane that visits i, i + Dw, i + 2 Dw, ... stays in one cell for about 1 / |sigma(Dw)|
// visits and makes d / Dw visits in all, so it issues about  d/Dw * |sigma| + 1  atomic adds for
// d / Dw coordinates: |sigma(Dw)| + Dw / d per coordinate.  The plan minimises that sum over all
// Dw up to d / 2 by brute force.
void plan_walk(cs_row_plan* rp, uint64_t a, uint64_t as, uint32_t c, bool pow2, uint64_t d_hint) {
    uint64_t best_D = 1;
    if (pow2 && c >= 64) {
        const uint64_t d_eff = d_hint ? d_hint : 64ull * c;
        const uint64_t d_max = d_eff / 2 < kPlanScanMax ? d_eff / 2 : kPlanScanMax;
        double best_cost = 1e300;
        uint64_t x = 0;                                 // (a * D) mod p
        const double inv_p = 1.0 / (double)kP61, inv_d = 1.0 / (double)d_eff;
        for (uint64_t D = 1; D <= d_max; ++D) {
            x += a;
            if (x >= kP61) x -= kP61;
            double adv = (double)(x & (c - 1)) + (double)x * inv_p;   // [0, c + 1)
            if (adv > 0.5 * c) adv -= (double)c;
            if (adv < 0) adv = -adv;
            const double cost = adv + (double)D * inv_d;
            if (cost < best_cost) { best_cost = cost; best_D = D; }
        }
    }
    rp->Dw = best_D;
    rp->ADw = mulmod(a, rp->Dw);
    rp->ADws = mulmod(as, rp->Dw);
}

// Estimated time, in nanoseconds, of one launch of the bundle update for a group of 8 workers:
// `visits` turns of the busiest wavefront in a row (each costs about kVisitNs of latency that
// nothing hides when few wavefronts are resident), stretched when there are more wavefronts
// than the chip holds at once; never less than reading the 8 vectors at the rate this access
// pattern reaches; plus the atomic requests at the rate of the memory-side atomic unit.  The
// constants are measurements on MI355X (bundle update at d = 10^6 .. 10^8).
double update_time_ns(double visits, double residues, double requests, double d) {
    const double kVisitNs = 900.0, kResidentWaves = 4096.0;
    const double kBytesPerNs = 4600.0, kRequestsPerNs = 24.0;
    const double waves = residues / 128.0;
    double serial = visits * kVisitNs;
    if (waves > kResidentWaves) serial *= waves / kResidentWaves;
    const double stream = d * 32.0 / kBytesPerNs;
    return (serial > stream ? serial : stream) + requests / kRequestsPerNs;
}

// Visit list of the bundle update for one row (cs_visit_plan).
//
// Rotating a hash value left by sh = 61 - log2(c) bits is a multiplication by 2^sh mod p, so
// u(i) = rot(a i + b) is again affine in i, its top bits are the bucket, and moving s
// coordinates on adds exactly U(s) = (s * U(1)) mod p.  For a bound omega (in cells) the list
// is { s < d : U(s) < omega * 2^sh } together with s = 0: every visit of a lane then lands
// in one of ncell = ceil(omega) + 1 neighbouring cells, whose sums it keeps in registers.
// Lanes own the residues [0, gmax), gmax the largest gap between neighbouring list entries,
// so a worker group sends about ncell * gmax requests for the whole vector, in K visits.  A
// wide bound means many visits and few requests, a narrow one the opposite; the bound is
// chosen by the time model above (one scan of s = 1 .. d - 1 collects the candidates for the
// widest bound, narrower ones are subsets).
void plan_visits(cs_visit_plan* vp, const cs_row_plan* rp, uint64_t a, uint64_t as, uint32_t c,
                 bool pow2, uint64_t d_hint) {
    memset(vp, 0, sizeof(*vp));
    if (!pow2 || c < 64 || d_hint < 4096 || d_hint > kPlanScanMax) return;
    int lc = 0;
    while ((1u << lc) < c) ++lc;
    const int sh = 61 - lc;
    const uint64_t cell = 1ull << sh;
    const uint64_t u1 = mulmod(a, cell % kP61);            // U(1)
    // the stride walk's requests, for comparison: d (|sigma(Dw)| + Dw / d)
    {
        const uint64_t Uw = mulmod(u1, rp->Dw % kP61);
        const uint64_t mag = Uw < kP61 - Uw ? Uw : kP61 - Uw;
        const double requests = (double)d_hint * ((double)mag / (double)cell) + (double)rp->Dw;
        vp->cost_walk = (uint64_t)update_time_ns((double)d_hint / (double)rp->Dw, (double)rp->Dw,
                                                 requests, (double)d_hint);
    }
    const double per_cell = (double)d_hint / (double)c;    // list entries per cell of bound
    double omega_max = (CS_MAX_VISITS - 16) / per_cell;
    if (omega_max > 3.0) omega_max = 3.0;
    if (omega_max * per_cell < 8.0) return;                // too few visits to pay off
    const uint64_t U_max = (uint64_t)(omega_max * (double)cell);
    std::vector<uint64_t> cs_, cu_;                        // candidate offsets and their U
    {
        uint64_t u = 0;
        for (uint64_t s = 1; s < d_hint; ++s) {
            u += u1;
            if (u >= kP61) u -= kP61;
            if (u < U_max) {
                cs_.push_back(s);
                cu_.push_back(u);
                if (cs_.size() > 16 * CS_MAX_VISITS) return;   // not a rotation-like row: give up
            }
        }
    }
    uint64_t best_cost = ~0ull, best_bound = 0;
    constexpr int kGrid = 96;
    for (int t = 1; t <= kGrid; ++t) {
        const uint64_t bound = (uint64_t)((double)U_max * t / kGrid);
        if (bound == 0) continue;
        uint64_t prev = 0, gmax = 0, K = 1;
        for (size_t q = 0; q < cs_.size(); ++q)
            if (cu_[q] < bound) {
                if (cs_[q] - prev > gmax) gmax = cs_[q] - prev;
                prev = cs_[q];
                ++K;
            }
        if (d_hint - prev > gmax) gmax = d_hint - prev;
        if (K < 4 || K > CS_MAX_VISITS) continue;
        const uint64_t ncell = ((bound + cell - 1) >> sh) + 1;
        const uint64_t cost = (uint64_t)update_time_ns((double)K, (double)gmax,
                                                       (double)(ncell * gmax), (double)d_hint);
        if (cost < best_cost) { best_cost = cost; best_bound = bound; }
    }
    if (best_bound == 0) return;
    // build the list for the chosen bound
    uint64_t gaps[3], prev = 0;
    int ngap = 0;
    uint32_t K = 0;
    auto add_visit = [&](uint64_t gap, bool last) -> bool {
        int code = 3;
        if (!last) {
            for (code = 0; code < ngap; ++code)
                if (gaps[code] == gap) break;
            if (code == ngap) {
                if (ngap == 3) return false;               // more than three return times
                gaps[ngap++] = gap;
            }
        }
        vp->code[K / 16] |= (uint32_t)code << (2 * (K % 16));
        ++K;
        return true;
    };
    for (size_t q = 0; q < cs_.size(); ++q)
        if (cu_[q] < best_bound) {
            if (!add_visit(cs_[q] - prev, false)) { memset(vp->code, 0, sizeof(vp->code)); return; }
            prev = cs_[q];
        }
    add_visit(d_hint - prev, true);
    for (int q = 0; q < 4; ++q) {
        const uint64_t gap = q < ngap ? gaps[q] : (q == 3 ? d_hint - prev : 0);
        vp->gap[q] = gap;
        vp->A[q] = mulmod(a, gap % kP61);
        vp->As[q] = mulmod(as, gap % kP61);
        if (gap > vp->gmax) vp->gmax = gap;
    }
    vp->ncell = (uint32_t)(((best_bound + cell - 1) >> sh) + 1);
    vp->cover = d_hint;
    vp->cost = best_cost;
    vp->K = K;
}

// Visit list for a column count that is not a power of two (cs_anyc_plan).
//
// One scan of s = 1 .. d - 1 keeps x = (a s) mod p and x mod c side by side (both step by a
// constant, minus p resp. p mod c on a wrap, so no division is needed) and collects the offsets
// whose x mod c is 0 or 1.  For omega = 1 and 2 and a few target gaps T, visits are then picked
// greedily: the last qualifying offset within T of the previous visit, or, if there is none,
// the first one beyond.  The list with the lowest estimated time (same model as for the
// power-of-two lists, 2 omega requests per residue) is kept if it beats one request per
// coordinate.
void plan_anyc(cs_anyc_plan* vp, uint64_t a, uint32_t c, bool pow2, uint64_t d_hint) {
    memset(vp, 0, sizeof(*vp));
    if (pow2 || c < 64 || d_hint < 65536 || d_hint > kPlanScanMax) return;
    const uint64_t ac = a % c, pc = kP61 % c;
    std::vector<uint32_t> pos[2];                          // offsets with x mod c == 0, == 1
    {
        uint64_t x = 0, r = 0;
        for (uint64_t s = 1; s < d_hint; ++s) {
            x += a;
            r += ac;
            if (r >= c) r -= c;
            if (x >= kP61) {
                x -= kP61;
                r = r >= pc ? r - pc : r + c - pc;
            }
            if (r < 2) {
                pos[r].push_back((uint32_t)s);
                if (pos[0].size() + pos[1].size() > (4u << 20)) return;    // c far too small for d
            }
        }
    }
    vp->cost_direct = (uint64_t)update_time_ns(1.0, 128.0, (double)d_hint, (double)d_hint);
    uint64_t best_cost = ~0ull;
    std::vector<uint32_t> best_gaps;
    uint32_t best_omega = 0;
    for (uint32_t omega = 1; omega <= 2; ++omega) {
        std::vector<uint32_t> q(pos[0]);
        if (omega == 2) {
            q.insert(q.end(), pos[1].begin(), pos[1].end());
            std::sort(q.begin(), q.end());
        }
        if (q.size() < 4) continue;
        for (uint32_t Kt : {12u, 16u, 24u, 32u, 48u, 64u, 96u, 128u, 143u}) {
            const uint64_t T = d_hint / Kt;
            if (T == 0) continue;
            std::vector<uint32_t> gaps;
            uint64_t prev = 0, gmax = 0;
            size_t at = 0;                                 // first qualifying offset > prev
            bool ok = true;
            while (prev + T < d_hint) {
                while (at < q.size() && q[at] <= prev) ++at;
                if (at == q.size()) break;
                size_t pick = at;                          // the first one beyond, unless ...
                while (pick + 1 < q.size() && q[pick + 1] <= prev + T) ++pick;   // ... one lies within T
                const uint64_t next = q[pick];
                gaps.push_back((uint32_t)(next - prev));
                if (next - prev > gmax) gmax = next - prev;
                prev = next;
                if (gaps.size() >= CS_ANYC_MAX_VISITS) { ok = false; break; }
            }
            if (!ok) continue;
            gaps.push_back((uint32_t)(d_hint - prev));
            if (d_hint - prev > gmax) gmax = d_hint - prev;
            if (gaps.size() < 4) continue;
            const uint64_t cost = (uint64_t)update_time_ns((double)gaps.size(), (double)gmax,
                                                           2.0 * omega * (double)gmax, (double)d_hint);
            if (cost < best_cost) { best_cost = cost; best_gaps = gaps; best_omega = omega; }
        }
    }
    if (best_gaps.empty()) return;
    vp->K = (uint32_t)best_gaps.size();
    vp->omega = best_omega;
    vp->cover = d_hint;
    vp->cost = best_cost;
    for (size_t k = 0; k < best_gaps.size(); ++k) {
        vp->gap[k] = best_gaps[k];
        if (best_gaps[k] > vp->gmax) vp->gmax = best_gaps[k];
    }
}

}  // namespace

extern "C" int cs_params_init(cs_params* p, uint32_t r, uint32_t c, uint64_t seed,
                              int64_t d_hint) {
    if (!p) return CS_EINVAL;
    if (r == 0 || r > CS_MAX_R || (r & 1u) == 0) return CS_EINVAL;
    if (c == 0 || c > (1u << 31)) return CS_EINVAL;
    if ((uint64_t)r * c > 0xffffffffull) return CS_EINVAL;   // cell indices are 32-bit
    if (d_hint < 0) return CS_EINVAL;
    memset(p, 0, sizeof(*p));
    p->r = r;
    p->c = c;
    p->c_pow2 = (c & (c - 1)) == 0 ? 1u : 0u;
    p->seed = seed;
    uint64_t st = seed;
    for (uint32_t j = 0; j < r; ++j) {
        p->a[j] = 1 + splitmix64(&st) % (kP61 - 1);
        p->b[j] = splitmix64(&st) % kP61;
        p->as[j] = 1 + splitmix64(&st) % (kP61 - 1);
        p->bs[j] = splitmix64(&st) % kP61;
    }
    for (uint32_t j = 0; j < r; ++j)
    {
        plan_row(&p->plan[j], p->a[j], p->as[j], c, p->c_pow2 != 0, (uint64_t)d_hint);
        plan_walk(&p->plan[j], p->a[j], p->as[j], c, p->c_pow2 != 0, (uint64_t)d_hint);
        plan_visits(&p->visit[j], &p->plan[j], p->a[j], p->as[j], c, p->c_pow2 != 0,
                    (uint64_t)d_hint);
        plan_anyc(&p->anyc[j], p->a[j], c, p->c_pow2 != 0, (uint64_t)d_hint);
    }
    return CS_OK;
}

extern "C" const char* cs_status_string(int status) {
    switch (status) {
        case CS_OK: return "ok";
        case CS_EINVAL: return "invalid argument";
        case CS_EWORKSPACE: return "workspace too small";
        case CS_EHIP: return "HIP runtime error";
        case CS_ELIMIT: return "input exceeds the limit of this entry point's built-in scratch";
        default: return "unknown status";
    }
}
