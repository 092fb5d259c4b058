"""A short selection of the mutation check (tests/oracle_mutation_check.py holds the full list): one planted
mistake per part of the oracle -- env rule, draw layout, sampler tie, bf16 rounding point, returns, loss gradient,
clamp, Adam, V-trace, pathwise adjoint -- must each turn the pins red.  CPU only."""
import oracle_mutation_check as M

SELECTION = [
    "catch: ball before paddle",
    "maze: walls ignored",
    "rollout: reset draw = action draw",
    "sample: cdf strict",
    "fp64: head weights unrounded",
    "returns: lambda mix",
    "loss: gauss clamp ignored",
    "adam: eps inside sqrt",
    "vtrace: gaussian ratio clamp",
    "path: obs adjoint sign",
]


def test_planted_mistakes_in_the_oracle_are_caught():
    names = {n for n, _, _ in M.MUTATIONS}
    assert set(SELECTION) <= names
    assert M.run(SELECTION, jobs=4) == []
