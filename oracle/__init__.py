"""CPU oracle of the linear-angular attention layer (test infrastructure only).

Only tests/, the smoke check and the bench's cpu_baseline leg may import this
package; the product path never does.
"""
from .castling_oracle import *  # noqa: F401,F403
