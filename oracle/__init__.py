"""CPU oracle of the DSLA layer forward.  Test infrastructure only: nothing in the
product package imports this, and this imports nothing from the product package."""
