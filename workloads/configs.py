"""The five workload shapes the query path is exercised on.

Symbols follow the paper: D vector dimension, P tree parts, k1/k2 first- and
second-level centroids per part (Sec. 3.1), w first-level clusters refined per
part (Sec. 3.2), M re-ranking sub-parts ("P_line", Sec. 3.3, last paragraph),
H number of (hashed) bin slots (Sec. 4), T bin tuples examined per query,
C candidate budget per query, k results per query.
"""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    kind: str          # generator family: "tiny" | "sift" | "gist"
    N: int             # database vectors
    D: int
    nq: int            # queries
    P: int
    k1: int
    k2: int
    M: int             # code bytes per vector
    H: int             # bin slots (== (k1*k2)**P when not hashed)
    T: int
    C: int
    k: int
    w: int
    train_n: int       # vectors the codebooks are trained on (the first train_n)
    data_seed: int = 0
    query_seed: int = 1

    @property
    def K(self) -> int:
        return (self.k1 * self.k2) ** self.P

    def with_(self, **kw) -> "WorkloadConfig":
        return replace(self, **kw)


CONFIGS = {
    # small enough for the oracle plus brute force to finish in seconds
    "tiny": WorkloadConfig("tiny", "tiny", N=10_000, D=32, nq=100, P=2, k1=8, k2=4, M=4,
                           H=(8 * 4) ** 2, T=64, C=256, k=10, w=2, train_n=10_000),
    # SIFT1M-shaped (Sec. 5, Table 1): the configuration the headline metric is quoted on
    "sift": WorkloadConfig("sift", "sift", N=1_000_000, D=128, nq=10_000, P=2, k1=16, k2=8, M=8,
                           H=(16 * 8) ** 2, T=1024, C=4096, k=100, w=8, train_n=100_000),
    # GIST1M-shaped (Sec. 5, Table 2)
    "gist": WorkloadConfig("gist", "gist", N=1_000_000, D=960, nq=1_000, P=4, k1=16, k2=8, M=16,
                           H=(16 * 8) ** 4, T=4096, C=4096, k=100, w=4, train_n=100_000),
    # 100M SIFT-shaped vectors held only as codes + inverted lists
    "large": WorkloadConfig("large", "sift", N=100_000_000, D=128, nq=10_000, P=2, k1=32, k2=16, M=8,
                            H=(32 * 16) ** 2, T=1024, C=10_000, k=100, w=8, train_n=1_000_000),
    # SIFT1B-shaped (Sec. 5.1, Fig. 6)
    "billion": WorkloadConfig("billion", "sift", N=1_000_000_000, D=128, nq=10_000, P=2, k1=64, k2=16,
                              M=8, H=(64 * 16) ** 2, T=1024, C=10_000, k=100, w=8, train_n=1_000_000),
    # the tree the paper itself uses at this scale (Sec. 5.1): four parts, bin numbers hashed by a plain
    # modulus to a prime number of slots near N/10 (collisions share a list)
    "large4": WorkloadConfig("large4", "sift", N=100_000_000, D=128, nq=10_000, P=4, k1=32, k2=16, M=8,
                             H=10_000_019, T=1024, C=10_000, k=100, w=8, train_n=1_000_000),
    "billion4": WorkloadConfig("billion4", "sift", N=1_000_000_000, D=128, nq=10_000, P=4, k1=32, k2=16,
                               M=8, H=100_000_007, T=1024, C=10_000, k=100, w=8, train_n=1_000_000),
}


def get_config(name: str) -> WorkloadConfig:
    return CONFIGS[name]
