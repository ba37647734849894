"""Where the vector work of a wide iteration stands between its MFMAs (the tables in csrc/attn_kernels.hip).

A wide unit runs one wavefront per SIMD, which issues in order: an MFMA that finds the matrix pipe busy holds up
everything behind it, and a gap with more than about 26 cycles of other instructions leaves the pipe idle.  An
iteration has 32 MFMAs (sixteen chunks of two) and so 32 gaps; gap 2c is behind the first MFMA of chunk c, gap
2c + 1 behind the second.  What a gap holds anyway:

  * gap 2c: the chunk's LDS request, one ds_read_b128 for a K fragment (chunks 0-3 and 12-15) or two transposing
    reads for a V fragment (chunks 4-11);
  * gap 2c + 1 for c + 1 in {4, 6, 8, 10, 12, 14}: the s_waitcnt in front of the next even chunk;
  * gap 2c + 1 for c in {1, 5, 9, 13}: one LDS-direct K/V load (with its M0 set-up);
  * gap 31: the end of the iteration (branch, loop bookkeeping).

The 32 exponentials (one per score of the lane), 16 bf16 packings (one per pair of exponentials) and 32 row-sum
additions are dealt out over the gaps so that every gap costs about the same, with issue costs measured for a
lone wavefront (the library's xy_probe_issue_mix shows the same figures): exp2 8.5 cycles, other vector
instructions 5, an LDS request 5.7, a wait 4.7.  A packing or an addition stands in a later gap than the
exponentials it reads, so that no wait state is padded between them.

    python -m paper_2412_18106_amd.gap_tables        prints the three tables as C initialisers

tables() returns cumulative counts: entry k = how many are done before gap k (33 entries each).
"""
from __future__ import annotations

COST_EXP, COST_VALU, COST_LDS, COST_WAIT, COST_LOAD, COST_LOOP_END = 8.5, 5.0, 5.7, 4.7, 16.0, 18.0
N_GAPS, N_EXP, N_CVT, N_ADD = 32, 32, 16, 32
GAP_CAP, SLACK, EXP_LEAD = 26.5, 6.0, 4      # most a gap may hold; how far ahead of an even pace; exponentials ahead of their readers


def fixed_cost(gap):
    chunk, second = divmod(gap, 2)
    cost = 0.0
    if not second:
        cost += COST_LDS if (chunk < 4 or chunk >= 12) else 2 * COST_LDS
    else:
        if chunk + 1 in (4, 6, 8, 10, 12, 14):
            cost += COST_WAIT
        if chunk & 3 == 1:
            cost += COST_LOAD
        if gap == N_GAPS - 1:
            cost += COST_LOOP_END
    return cost


def tables():
    total = N_EXP * COST_EXP + (N_CVT + N_ADD) * COST_VALU + sum(fixed_cost(g) for g in range(N_GAPS))
    exp_done = cvt_done = add_done = 0
    k_exp, k_cvt, k_add = [0], [0], [0]
    spent = 0.0
    for gap in range(N_GAPS):
        # what the iteration should have spent by the end of this gap if every gap cost the same
        goal = total * (gap + 1) / N_GAPS
        here = fixed_cost(gap)
        exp_before = exp_done               # consumers in this gap read exponentials of earlier gaps only
        last = gap == N_GAPS - 1

        def fits(cost):
            return last or (here + cost <= GAP_CAP and spent + here + cost <= goal + SLACK)

        while True:
            ready_cvt = cvt_done < N_CVT and 2 * cvt_done + 2 <= exp_before
            ready_add = add_done < N_ADD and add_done + 1 <= exp_before
            # the exponentials keep a lead over their consumers (they unlock everything else) ...
            lead = exp_done - max(2 * cvt_done, add_done)
            if exp_done < N_EXP and lead < EXP_LEAD and fits(COST_EXP):
                exp_done += 1
                here += COST_EXP
            # ... then whatever is ready, oldest pair first
            elif (ready_cvt or ready_add) and fits(COST_VALU):
                if ready_cvt and (not ready_add or 2 * cvt_done < add_done):
                    cvt_done += 1
                else:
                    add_done += 1
                here += COST_VALU
            elif exp_done < N_EXP and fits(COST_EXP):
                exp_done += 1
                here += COST_EXP
            else:
                break
        spent += here
        k_exp.append(exp_done)
        k_cvt.append(cvt_done)
        k_add.append(add_done)
    assert (exp_done, cvt_done, add_done) == (N_EXP, N_CVT, N_ADD), (exp_done, cvt_done, add_done)
    return k_exp, k_cvt, k_add


def gap_costs(k_exp, k_cvt, k_add):
    return [fixed_cost(g) + COST_EXP * (k_exp[g + 1] - k_exp[g])
            + COST_VALU * (k_cvt[g + 1] - k_cvt[g] + k_add[g + 1] - k_add[g]) for g in range(N_GAPS)]


def check(k_exp, k_cvt, k_add):
    """The rules a table must obey whatever made it: monotone, complete, and no consumer in or before the gap of
    an exponential it reads."""
    for t, n in ((k_exp, N_EXP), (k_cvt, N_CVT), (k_add, N_ADD)):
        assert len(t) == N_GAPS + 1 and t[0] == 0 and t[-1] == n and all(a <= b for a, b in zip(t, t[1:]))
    for g in range(N_GAPS):
        assert 2 * k_cvt[g + 1] <= k_exp[g], f"a packing in gap {g} reads an exponential of the same gap"
        assert k_add[g + 1] <= k_exp[g], f"an addition in gap {g} reads an exponential of the same gap"


def as_c(table):
    return "{" + ", ".join(str(x) for x in table) + "}"


if __name__ == "__main__":
    ke, kc, ka = tables()
    check(ke, kc, ka)
    print("#define XY_GAP_TABLE_EXP " + as_c(ke))
    print("#define XY_GAP_TABLE_CVT " + as_c(kc))
    print("#define XY_GAP_TABLE_ADD " + as_c(ka))
    print("// cycles per gap:", " ".join(f"{c:.0f}" for c in gap_costs(ke, kc, ka)))
