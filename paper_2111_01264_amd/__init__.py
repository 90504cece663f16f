"""MI355X-native DQN hot path (replay gather, batched act step, minibatch train step) behind a
C-ABI library; this package is its thin Python binding."""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTS, LIB_PATH, DqnError, dqn_config  # noqa: F401
