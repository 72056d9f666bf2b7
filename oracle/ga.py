"""Step-by-step genetic search oracle.  TEST INFRASTRUCTURE ONLY.

Follows Section 2.3 "Genetic search" of the paper in its own order and notation:

* a configuration is a chromosome ``s = {c_0 .. c_{n-1}}`` of integer genes, each with a
  finite range ("Search space");
* Step1 draws ``|a|`` random chromosomes and keeps only those that pass the constraint check;
* Step2 gives every individual a fitness ``f(a_i)``, a function of its measured runtime;
* Step3 turns fitness into selection probabilities ``p(a_i) = f(a_i) / sum_j f(a_j)`` (eq. 1),
  sorts by decreasing probability, passes the top ``k`` elites on unchanged and breeds the
  remaining ``|a'| - k`` children from parents picked by roulette wheel: cumulative
  probabilities ``P(a_i) = sum_{j<=i} p(a_j)`` over the ``m`` participating individuals
  (eq. 2), a uniform ``v``, and the individual ``i`` with ``P(a_{i-1}) < v <= P(a_i)``;
* Step4 repeats Step2-3 until the runtimes within a generation are close enough.

Readings where the paper is silent (each also listed in the design document):

* fitness is ``1 / runtime`` (larger is better; the elites are the "highest probabilities");
  an individual that cannot run has fitness 0;
* the ``m`` participants are the ``m`` fittest, and ``p`` is re-normalised over them so that
  ``P(a_m) = 1``; ``P(a_0) = 0`` and ``v = 0`` selects the first individual; if every
  participant has fitness 0 they are equally likely;
* crossover is uniform (each gene from the first parent with probability 1/2, else from the
  second); mutation re-draws each gene uniformly in its range with probability ``pm``;
  a child that fails the constraint check is bred again (``retries`` times), then replaced by
  a fresh random legal chromosome;
* chromosomes already evaluated reuse their fitness;
* "close enough": every runtime of the generation within ``eps`` (relative) of the fastest,
  or no improvement of the best for ``patience`` generations, or ``max_gen`` generations;
* all random numbers come from one splitmix64 stream (Steele, Lea, Flood 2014), consumed in
  the order the steps above are written.  The HIP library's host-side search engine
  implements the same generator on its own, so that both sides can be compared generation
  by generation; no code is shared.

Pure Python on purpose: sums run left to right in the sorted order, as eq. (1)-(2) read.
"""

MASK64 = (1 << 64) - 1


class SplitMix64:
    """splitmix64: state += golden gamma; output = finalising mix of the state."""

    def __init__(self, seed):
        self.state = seed & MASK64

    def next_u64(self):
        self.state = (self.state + 0x9E3779B97F4A7C15) & MASK64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
        return z ^ (z >> 31)

    def uniform(self):
        """53-bit uniform in [0, 1)."""
        return (self.next_u64() >> 11) * (1.0 / 9007199254740992.0)

    def randint(self, lo, hi):
        """Integer in [lo, hi] (plain modulo reduction of one 64-bit draw)."""
        return lo + self.next_u64() % (hi - lo + 1)


def selection_probabilities(fitness):
    """Eq. (1): p(a_i) = f(a_i) / sum_j f(a_j).  All-zero fitness gives equal probabilities."""
    total = 0.0
    for f in fitness:
        total += f
    if total <= 0.0:
        return [1.0 / len(fitness)] * len(fitness)
    return [f / total for f in fitness]


def cumulative_probabilities(p):
    """Eq. (2): P(a_i) = sum_{j<=i} p(a_j); the last entry is forced to exactly 1."""
    out, run = [], 0.0
    for v in p:
        run += v
        out.append(run)
    out[-1] = 1.0
    return out


def roulette_pick(P, v):
    """Inverse sampling: the (0-based) index i with P[i-1] < v <= P[i], where P[-1] = 0.
    v = 0 picks the first individual."""
    for i, Pi in enumerate(P):
        if v <= Pi:
            return i
    return len(P) - 1


def sort_by_fitness(fitness):
    """Indices in decreasing fitness; ties keep population order."""
    return sorted(range(len(fitness)), key=lambda i: (-fitness[i], i))


def random_legal(rng, lo, hi, constraint, max_tries=100000):
    for _ in range(max_tries):
        chrom = tuple(rng.randint(l, h) for l, h in zip(lo, hi))
        if constraint(chrom):
            return chrom
    raise RuntimeError("no legal chromosome found")


def breed(rng, parents, P, lo, hi, constraint, pm, retries):
    """One child: two roulette parents, uniform crossover, per-gene mutation."""
    for _ in range(retries):
        a = parents[roulette_pick(P, rng.uniform())]
        b = parents[roulette_pick(P, rng.uniform())]
        child = [a[g] if rng.uniform() < 0.5 else b[g] for g in range(len(lo))]
        for g in range(len(lo)):
            if rng.uniform() < pm:
                child[g] = rng.randint(lo[g], hi[g])
        child = tuple(child)
        if constraint(child):
            return child
    return random_legal(rng, lo, hi, constraint)


def next_generation(rng, population, fitness, lo, hi, constraint, k, m, next_size, pm, retries):
    """Step3 for one generation.  Returns the new population (elites first)."""
    order = sort_by_fitness(fitness)
    elites = [population[i] for i in order[:k]]
    part = order[:m]
    parents = [population[i] for i in part]
    P = cumulative_probabilities(selection_probabilities([fitness[i] for i in part]))
    children = [breed(rng, parents, P, lo, hi, constraint, pm, retries)
                for _ in range(next_size - k)]
    return elites + children


def runtimes_close(fitness, eps):
    """Step4 test: all individuals ran, and the slowest is within eps of the fastest."""
    if any(f <= 0.0 for f in fitness):
        return False
    t = [1.0 / f for f in fitness]
    return (max(t) - min(t)) / min(t) < eps


def genetic_search(lo, hi, constraint, fitness_fn, seed, pop=32, elites=4, next_pop=None,
                   participants=None, pm=0.1, retries=8, eps=0.05, patience=5, max_gen=20):
    """Run Steps 1-4.  Returns a dict with the best chromosome, its fitness, the number of
    fitness evaluations, and ``history`` = [(population, fitness list)] per generation."""
    next_pop = pop if next_pop is None else next_pop
    rng = SplitMix64(seed)
    memo = {}

    def evaluate(ch):
        if ch not in memo:
            memo[ch] = float(fitness_fn(ch))
        return memo[ch]

    population = [random_legal(rng, lo, hi, constraint) for _ in range(pop)]  # Step1
    history, best, best_f, stall = [], None, -1.0, 0
    for gen in range(max_gen):
        fit = [evaluate(ch) for ch in population]                              # Step2
        history.append((list(population), list(fit)))
        top = sort_by_fitness(fit)[0]
        if fit[top] > best_f:
            best, best_f, stall = population[top], fit[top], 0
        else:
            stall += 1
        if runtimes_close(fit, eps) or stall >= patience or gen == max_gen - 1:  # Step4
            break
        m = len(population) if participants is None else min(participants, len(population))
        population = next_generation(rng, population, fit, lo, hi, constraint,       # Step3
                                     min(elites, len(population)), m, next_pop, pm, retries)
    return {"best": best, "best_fitness": best_f, "evaluations": len(memo), "history": history}
