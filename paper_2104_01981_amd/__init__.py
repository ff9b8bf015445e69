"""MI355X-native ECRM parameter-server update path: Python binding of the C-ABI library."""
from .binding import (  # noqa: F401
    ECRM_EBATCH, ECRM_EBUFFER, ECRM_EHIP, ECRM_ESTATE, ECRM_EINVAL, ECRM_EKEYRANGE, ECRM_ENOTBOUND, ECRM_ESCRATCH, ECRM_OK,
    ECRM_PHASES, EcrmConfig, EcrmError, Ecrm, library_path, load_library, probe_row_traffic,
)
