"""MI355X-native forward + BPTT for generalized LSTM-like RNN graphs (C-ABI library + binding)."""
from .binding import Graph, RnnError, load_library, LIB_PATH, EXPORTS, AUX_EXPORTS  # noqa: F401
