"""Time-to-accuracy on the synthetic quadratic under the paper's timing model.

The paper's end-to-end figure of merit (Section 5: training time until a target accuracy) is
iterations-to-accuracy times the average iteration time T_avg.  Here the iterations come from
the DD-EF-SGD path on the GPU (Algorithm 1 on the synthetic objective of problem (1)), and T_avg
from the pipeline recurrence of Section 4.1 / Theorem 3 for a network of bandwidth a and latency
b.  `strategies` names the corners of the (tau, delta) plane: D-SGD (tau = 0, delta = 1),
compression only, delay only, and DeCo's joint choice (Algorithm 3); every (tau, delta) comes from
the library (ddef_corner_*, ddef_deco), this module only runs them.

    python -m paper_2507_17346_amd.time_to_accuracy --d 1000000 --n 4 --a-mbps 100 --b 0.2
"""
import argparse
from dataclasses import dataclass
from typing import List, Optional, Tuple

from . import binding, workloads


@dataclass(frozen=True)
class Network:
    v_g_bits: float      # size of an uncompressed gradient, bits
    a_bps: float         # bandwidth, bits per second
    b_s: float           # end-to-end latency, seconds
    t_comp_s: float      # computation time of one iteration, seconds


@dataclass(frozen=True)
class Strategy:
    name: str
    tau: int
    delta: float                         # ddef_ef_compress's ratio = share of V_g that crosses the wire


@dataclass
class Outcome:
    strategy: Strategy
    t_avg_s: float
    iterations: Optional[int]            # first checked iteration with f <= target, None if never
    seconds: Optional[float]
    curve: List[Tuple[int, float, float]]  # (iteration, seconds, f / f(x_0))


def strategies(net: Network, tau_max: int) -> List[Strategy]:
    """D-SGD; compression only and delay only (ddef_corner_*); DeCo (Algorithm 3), clamped to tau_max."""
    out = [Strategy("D-SGD", 0, 1.0)]
    out.append(Strategy("compression only", 0,
                        binding.corner_compression_only(net.v_g_bits, net.a_bps, net.t_comp_s)))
    out.append(Strategy("delay only",
                        binding.corner_delay_only(net.v_g_bits, net.a_bps, net.b_s, net.t_comp_s, tau_max), 1.0))
    chosen = binding.deco(net.v_g_bits, net.a_bps, net.b_s, net.t_comp_s)
    if chosen is not None:
        out.append(Strategy("DeCo", int(min(tau_max, chosen[0])), float(chosen[1])))
    return out


def t_avg(net: Network, s: Strategy, iterations: int = 2000) -> float:
    """Average iteration time of the pipeline of Section 4.1 (the recurrence, not the closed form)."""
    return binding.t_avg_simulate(s.tau, s.delta, net.v_g_bits, net.a_bps, net.b_s, net.t_comp_s, iterations)


def run(w, s: Strategy, net: Network, target_ratio: float, max_iterations: int, check_every: int,
        tau_max: Optional[int] = None) -> Outcome:
    """Runs DD-EF-SGD with (tau, delta) of `s` on workload `w` until f(x_t) <= target_ratio * f(x_0),
    looking every `check_every` iterations."""
    lam, xstar, x0 = workloads.make_problem(w)
    ctx = binding.Context(w.d, w.n, tau_max if tau_max is not None else max(s.tau, 1))
    try:
        ctx.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        ctx.set_tau(s.tau)
        per_iteration = t_avg(net, s)
        f0 = ctx.objective()
        curve = [(0, 0.0, 1.0)]
        reached = None
        t = 0
        while t < max_iterations and reached is None:
            for _ in range(check_every):
                ctx.step(s.delta, w.lr)
            t += check_every
            ratio = ctx.objective() / f0
            curve.append((t, t * per_iteration, ratio))
            if ratio <= target_ratio:
                reached = t
        return Outcome(s, per_iteration, reached, None if reached is None else reached * per_iteration, curve)
    finally:
        ctx.close()


def run_adaptive(w, nets: List[Network], period: int, adaptive: bool, target_ratio: float,
                 max_iterations: int, tau_max: int = 16, lut: Optional["binding.DecoLut"] = None) -> Outcome:
    """A network that changes every `period` iterations (nets[p % len(nets)] holds during period p).
    adaptive = True is DeCo-SGD (Algorithm 2): (tau, delta) re-chosen by Algorithm 3 at the start of
    every period from that period's network.  adaptive = False keeps the choice made for the
    first period.  Seconds accumulate period by period with each period's iteration time under
    the (tau, delta) in force; the objective is looked at once per period.  With `lut` (the look-up
    table of Section 4.5, built for one latency) the choice comes from the table entry nearest to the
    period's bandwidth instead of a run of Algorithm 3."""
    lam, xstar, x0 = workloads.make_problem(w)
    ctx = binding.Context(w.d, w.n, tau_max)
    try:
        ctx.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        f0 = ctx.objective()
        curve = [(0, 0.0, 1.0)]
        seconds, t, reached, p = 0.0, 0, None, 0
        first = None
        while t < max_iterations and reached is None:
            net = nets[p % len(nets)]
            if adaptive or first is None:
                choice = lut.query(net.a_bps) if lut is not None else binding.deco(
                    net.v_g_bits, net.a_bps, net.b_s, net.t_comp_s)
                if choice is None and first is None:
                    raise ValueError("Algorithm 3 has no candidate (tau, delta) for the first period's network")
                if choice is not None:             # no candidate for this network: the choice in force stays
                    first = Strategy("DeCo-SGD" if adaptive else "DeCo, first period's choice kept",
                                     int(min(tau_max, choice[0])), float(choice[1]))
            ctx.set_tau(first.tau)
            for _ in range(period):
                ctx.step(first.delta, w.lr)
            t += period
            seconds += period * t_avg(net, first, max(period, 2))
            ratio = ctx.objective() / f0
            curve.append((t, seconds, ratio))
            if ratio <= target_ratio:
                reached = t
            p += 1
        return Outcome(first, seconds / max(t, 1), reached, None if reached is None else seconds, curve)
    finally:
        ctx.close()


def compare(w, net: Network, target_ratio: float = 0.02, max_iterations: int = 20000, check_every: int = 50,
            tau_max: int = 16) -> List[Outcome]:
    return [run(w, s, net, target_ratio, max_iterations, check_every, tau_max) for s in strategies(net, tau_max)]


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="C1")
    ap.add_argument("--d", type=int, default=None)
    ap.add_argument("--n", type=int, default=None)
    ap.add_argument("--a-mbps", type=float, default=100.0)
    ap.add_argument("--b", type=float, default=0.2, help="latency, seconds")
    ap.add_argument("--t-comp", type=float, default=0.02, help="computation time per iteration, seconds")
    ap.add_argument("--target", type=float, default=0.02, help="stop at f <= target * f(x_0)")
    ap.add_argument("--max-iterations", type=int, default=20000)
    ap.add_argument("--check-every", type=int, default=50)
    args = ap.parse_args()
    w = workloads.get(args.workload, d=args.d, n=args.n)
    net = Network(32.0 * w.d, args.a_mbps * 1e6, args.b, args.t_comp)
    outcomes = compare(w, net, args.target, args.max_iterations, args.check_every)
    base = outcomes[0].seconds
    print(f"{w.name}: d={w.d} n={w.n}; a={args.a_mbps} Mbps, b={args.b} s, T_comp={args.t_comp} s; "
          f"target f <= {args.target} f(x_0)")
    print(f"{'strategy':18s} {'tau':>4s} {'delta':>9s} {'T_avg s':>9s} {'iterations':>10s} {'seconds':>10s} {'vs D-SGD':>9s}")
    for o in outcomes:
        it = "-" if o.iterations is None else str(o.iterations)
        sec = "-" if o.seconds is None else f"{o.seconds:.2f}"
        sp = "-" if o.seconds is None or base is None else f"{base / o.seconds:.2f}x"
        print(f"{o.strategy.name:18s} {o.strategy.tau:4d} {o.strategy.delta:9.5f} {o.t_avg_s:9.4f} {it:>10s} {sec:>10s} {sp:>9s}")


if __name__ == "__main__":
    main()
